// The two subnets outside the transformer blocks (Sec. IV-A, "Full fine-tuning partition settings"):
// the patch embedding at the start and the pooling + classification layer at the end.  The patch
// projection and its weight gradient run on the GEMM kernels; what is here is the bandwidth-bound
// data movement around them and the small per-image arithmetic of the classifier.
#include "d2ft_common.h"

namespace d2ft {

namespace {

// ---------------------------------------------------------------------------
// images [B][C][H][W] -> patches [B * ny * nx][C * P * P], k = (c * P + i) * P + j; 8 pixels of one
// image row per thread (P is a multiple of 8)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void im2col_kernel(const T* __restrict__ img, T* __restrict__ patches, int B, int C,
                                                     int H, int W, int P) {
    const int nx = W / P, ny = H / P, K = C * P * P, k8 = K / 8;
    const long total = (long)B * ny * nx * k8;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int kc = (int)(i % k8);
        const long row = i / k8;                    // b * ny * nx + py * nx + px
        const int px = (int)(row % nx), py = (int)((row / nx) % ny), b = (int)(row / ((long)nx * ny));
        const int k = kc * 8, c = k / (P * P), ii = (k / P) % P, j = k % P;
        float v[8];
        load8(img + (((long)b * C + c) * H + py * P + ii) * W + px * P + j, v);
        store8(patches + row * K + k, v);
    }
}

// tokens[b][0] = cls + pos[0]; tokens[b][1 + p] = proj[b * Np + p] + pos[1 + p]
template <typename T>
__global__ __launch_bounds__(256) void assemble_tokens_kernel(const T* __restrict__ proj, const T* __restrict__ cls,
                                                              const T* __restrict__ pos, T* __restrict__ tokens, int B,
                                                              int Np, int D) {
    const int d8 = D / 8, Tn = Np + 1;
    const long total = (long)B * Tn * d8;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
        const int dc = (int)(i % d8) * 8;
        const long row = i / d8;
        const int t = (int)(row % Tn), b = (int)(row / Tn);
        float a[8], p[8];
        if (t == 0) load8(cls + dc, a); else load8(proj + ((long)b * Np + t - 1) * D + dc, a);
        load8(pos + (long)t * D + dc, p);
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] += p[j];
        store8(tokens + row * D + dc, a);
    }
}

// backward of the assembly: dproj[b * Np + p] = dtokens[b][1 + p]; dpos[t] = sum_b dtokens[b][t] (images added
// in index order); dcls = dpos[0].  One thread per (t, 8 channels).
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_gather_kernel(const T* __restrict__ dtokens, T* __restrict__ dproj,
                                                               T* g_pos, T* g_cls, int B, int Np, int D, int accumulate) {
    const int d8 = D / 8, Tn = Np + 1;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Tn * d8) return;
    const int dc = (i % d8) * 8, t = i / d8;
    float s[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) s[j] = 0.f;
    for (int b0 = 0; b0 < B; b0 += 4) {      // four images in flight
        float v[4][8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (b0 + q < B) load8(dtokens + ((long)(b0 + q) * Tn + t) * D + dc, v[q]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (b0 + q < B) {
                if (t > 0) store8(dproj + ((long)(b0 + q) * Np + t - 1) * D + dc, v[q]);
#pragma unroll
                for (int j = 0; j < 8; ++j) s[j] += v[q][j];
            }
        }
    }
    auto emit = [&](T* out) {
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = s[j];
        if (accumulate) {
            float old[8];
            load8(out, old);
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] += old[j];
        }
        store8(out, o);
    };
    if (g_pos) emit(g_pos + (long)t * D + dc);
    if (g_cls && t == 0) emit(g_cls + dc);
}

// ---------------------------------------------------------------------------
// classifier, one workgroup per image: LayerNorm of the class token, logits, softmax cross-entropy
// and its gradient with respect to the logits.  All arithmetic fp32.
//   xhat, h: [B][D] fp32; logits, dl: [B][n] fp32; loss_b: [B]
// ---------------------------------------------------------------------------
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

template <typename T>
__global__ __launch_bounds__(256) void classifier_fwd_kernel(const T* __restrict__ tokens, const T* __restrict__ ln_g,
                                                             const T* __restrict__ ln_b, const T* __restrict__ w_c,
                                                             const T* __restrict__ b_c, const int32_t* __restrict__ labels,
                                                             int Tn, int D, int n, float eps, float* __restrict__ xhat,
                                                             float* __restrict__ h, float* __restrict__ rstd_out,
                                                             float* __restrict__ logits, float* __restrict__ dl,
                                                             float* __restrict__ loss_b, int B) {
    __shared__ float red[4];
    const int b = blockIdx.x;
    const T* x = tokens + (long)b * Tn * D;
    float s = 0.f;
    for (int d = threadIdx.x; d < D; d += 256) s += ld<T>(x + d);
    const float mean = block_sum(s, red) / D;
    float q = 0.f;
    for (int d = threadIdx.x; d < D; d += 256) {
        const float c = ld<T>(x + d) - mean;
        q += c * c;
    }
    const float rstd = rsqrtf(block_sum(q, red) / D + eps);
    for (int d = threadIdx.x; d < D; d += 256) {
        const float xh = (ld<T>(x + d) - mean) * rstd;
        xhat[(long)b * D + d] = xh;
        h[(long)b * D + d] = xh * ld<T>(ln_g + d) + ld<T>(ln_b + d);
    }
    if (threadIdx.x == 0) rstd_out[b] = rstd;
    __syncthreads();
    // logits: one wavefront per class, lanes stride over the channels
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int c = wave; c < n; c += 4) {
        float acc = 0.f;
        for (int d = lane; d < D; d += 64) acc = fmaf(h[(long)b * D + d], ld<T>(w_c + (long)c * D + d), acc);
        acc = wave_sum(acc);
        if (lane == 0) logits[(long)b * n + c] = acc + ld<T>(b_c + c);
    }
    __syncthreads();
    float m = -INFINITY;
    for (int c = threadIdx.x; c < n; c += 256) m = fmaxf(m, logits[(long)b * n + c]);
    m = wave_max(m);
    __syncthreads();
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float e = 0.f;
    for (int c = threadIdx.x; c < n; c += 256) e += __expf(logits[(long)b * n + c] - m);
    const float lse = m + __logf(block_sum(e, red));
    const int label = labels[b];
    for (int c = threadIdx.x; c < n; c += 256) {
        const float p = __expf(logits[(long)b * n + c] - lse);
        dl[(long)b * n + c] = (p - (c == label ? 1.f : 0.f)) / B;
    }
    if (threadIdx.x == 0) loss_b[b] = lse - logits[(long)b * n + label];
}

// dh = dl W_c, LayerNorm backward of the class-token row, zeros in the image's other rows of dtokens
template <typename T>
__global__ __launch_bounds__(256) void classifier_bwd_kernel(const float* __restrict__ dl, const T* __restrict__ w_c,
                                                             const T* __restrict__ ln_g, const float* __restrict__ xhat,
                                                             const float* __restrict__ rstd, int Tn, int D, int n,
                                                             float* __restrict__ dh, T* __restrict__ dtokens) {
    __shared__ float red[4];
    const int b = blockIdx.x;
    float m1 = 0.f, m2 = 0.f;
    for (int d = threadIdx.x; d < D; d += 256) {
        float acc = 0.f;
        for (int c = 0; c < n; ++c) acc = fmaf(dl[(long)b * n + c], ld<T>(w_c + (long)c * D + d), acc);
        dh[(long)b * D + d] = acc;
        const float dg = acc * ld<T>(ln_g + d);
        m1 += dg;
        m2 += dg * xhat[(long)b * D + d];
    }
    m1 = block_sum(m1, red) / D;
    m2 = block_sum(m2, red) / D;
    const float rs = rstd[b];
    T* out = dtokens + (long)b * Tn * D;
    for (int d = threadIdx.x; d < D; d += 256) {
        const float dg = dh[(long)b * D + d] * ld<T>(ln_g + d);
        st<T>(out + d, rs * (dg - m1 - xhat[(long)b * D + d] * m2));
    }
    for (long i = D + threadIdx.x; i < (long)Tn * D; i += 256) out[i] = static_cast<T>(0.0f);
}

// parameter gradients and the mean loss: images added in index order
//   blockIdx.x < n: row c of dW_c and db_c[c]; the last workgroup: dln_g, dln_b and the loss
template <typename T>
__global__ __launch_bounds__(256) void classifier_param_grad_kernel(const float* __restrict__ dl, const float* __restrict__ h,
                                                                    const float* __restrict__ dh,
                                                                    const float* __restrict__ xhat,
                                                                    const float* __restrict__ loss_b, int B, int D, int n,
                                                                    T* g_w_c, T* g_b_c, T* g_ln_g, T* g_ln_b,
                                                                    float* __restrict__ loss, int accumulate) {
    auto emit = [&](T* p, float v) {
        if (accumulate) v += ld<T>(p);
        st<T>(p, v);
    };
    if ((int)blockIdx.x < n) {
        const int c = blockIdx.x;
        if (g_w_c) {
            for (int d = threadIdx.x; d < D; d += 256) {
                float acc = 0.f;
                for (int b = 0; b < B; ++b) acc = fmaf(dl[(long)b * n + c], h[(long)b * D + d], acc);
                emit(g_w_c + (long)c * D + d, acc);
            }
        }
        if (g_b_c && threadIdx.x == 0) {
            float acc = 0.f;
            for (int b = 0; b < B; ++b) acc += dl[(long)b * n + c];
            emit(g_b_c + c, acc);
        }
        return;
    }
    for (int d = threadIdx.x; d < D; d += 256) {
        float a = 0.f, s = 0.f;
        for (int b = 0; b < B; ++b) {
            a = fmaf(dh[(long)b * D + d], xhat[(long)b * D + d], a);
            s += dh[(long)b * D + d];
        }
        if (g_ln_g) emit(g_ln_g + d, a);
        if (g_ln_b) emit(g_ln_b + d, s);
    }
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int b = 0; b < B; ++b) t += loss_b[b];
        *loss = t / B;
    }
}

#define D2FT_HEAD_DISPATCH(dtype, ...) \
    if ((dtype) == D2FT_F32) {         \
        typedef float T;               \
        __VA_ARGS__                    \
    } else {                           \
        typedef bf16 T;                \
        __VA_ARGS__                    \
    }

inline unsigned grid_for(long items) {
    long g = (items + 255) / 256;
    return (unsigned)(g < 1 ? 1 : (g > 8192 ? 8192 : g));
}

}  // namespace

hipError_t launch_im2col(int dtype, const void* img, void* patches, int B, int C, int H, int W, int P, hipStream_t s) {
    const long items = (long)B * (H / P) * (W / P) * (C * P * P / 8);
    D2FT_HEAD_DISPATCH(dtype, hipLaunchKernelGGL(im2col_kernel<T>, dim3(grid_for(items)), dim3(256), 0, s, (const T*)img,
                                                 (T*)patches, B, C, H, W, P);)
    return hipGetLastError();
}

hipError_t launch_assemble_tokens(int dtype, const void* proj, const void* cls, const void* pos, void* tokens, int B, int Np,
                                  int D, hipStream_t s) {
    const long items = (long)B * (Np + 1) * (D / 8);
    D2FT_HEAD_DISPATCH(dtype, hipLaunchKernelGGL(assemble_tokens_kernel<T>, dim3(grid_for(items)), dim3(256), 0, s,
                                                 (const T*)proj, (const T*)cls, (const T*)pos, (T*)tokens, B, Np, D);)
    return hipGetLastError();
}

hipError_t launch_embed_bwd_gather(int dtype, const void* dtokens, void* dproj, void* g_pos, void* g_cls, int B, int Np, int D,
                                   int accumulate, hipStream_t s) {
    const int items = (Np + 1) * (D / 8);
    D2FT_HEAD_DISPATCH(dtype, hipLaunchKernelGGL(embed_bwd_gather_kernel<T>, dim3((items + 255) / 256), dim3(256), 0, s,
                                                 (const T*)dtokens, (T*)dproj, (T*)g_pos, (T*)g_cls, B, Np, D, accumulate);)
    return hipGetLastError();
}

hipError_t launch_classifier(int dtype, const void* tokens, const void* ln_g, const void* ln_b, const void* w_c, const void* b_c,
                             const int32_t* labels, int B, int Tn, int D, int n, float eps, float* xhat, float* h, float* rstd,
                             float* logits, float* dl, float* loss_b, float* dh, void* dtokens, void* g_w_c, void* g_b_c,
                             void* g_ln_g, void* g_ln_b, float* loss, int accumulate, hipStream_t s) {
    D2FT_HEAD_DISPATCH(dtype,
        hipLaunchKernelGGL(classifier_fwd_kernel<T>, dim3(B), dim3(256), 0, s, (const T*)tokens, (const T*)ln_g, (const T*)ln_b,
                           (const T*)w_c, (const T*)b_c, labels, Tn, D, n, eps, xhat, h, rstd, logits, dl, loss_b, B);
        hipLaunchKernelGGL(classifier_bwd_kernel<T>, dim3(B), dim3(256), 0, s, dl, (const T*)w_c, (const T*)ln_g, xhat, rstd, Tn,
                           D, n, dh, (T*)dtokens);
        hipLaunchKernelGGL(classifier_param_grad_kernel<T>, dim3(n + 1), dim3(256), 0, s, dl, h, dh, xhat, loss_b, B, D, n,
                           (T*)g_w_c, (T*)g_b_c, (T*)g_ln_g, (T*)g_ln_b, loss, accumulate);)
    return hipGetLastError();
}

}  // namespace d2ft
