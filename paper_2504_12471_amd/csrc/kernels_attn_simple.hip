// Softmax attention forward and backward on the vector ALUs, one wavefront per query row
// (forward, dQ) or per key row (dK, dV).  Head dimension 64 = one lane per channel.  This is
// the fp32 path and the path for token counts the MFMA kernels do not take.  Probabilities are
// never stored: the backward pass rebuilds them from the saved log-sum-exp.
#include "d2ft_common.h"

namespace d2ft {

// dot product of a 64-vector held in LDS (fp32) with a 64-element row in global memory
template <typename T>
__device__ __forceinline__ float dot64(const float* __restrict__ a, const T* __restrict__ row) {
    float s = 0.f;
    float v[8];
#pragma unroll
    for (int c = 0; c < 64; c += 8) {
        load8(row + c, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) s = fmaf(a[c + i], v[i], s);
    }
    return s;
}

// grid (row_groups, batch * n_live); dynamic LDS: 4 * (64 + tokens) floats
template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simple_kernel(const T* __restrict__ qkv, long ldq, T* __restrict__ o,
                                                              long ldo, float* __restrict__ lse, int tokens,
                                                              int n_live, int n_full, long rows_total) {
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* qv = smem + wave * (64 + tokens);
    float* sc = qv + 64;
    const int b = blockIdx.y / n_live, j = blockIdx.y % n_live;
    const long row0 = (long)b * tokens;
    const T* Qb = qkv + row0 * ldq + j * 192;
    const T* Kb = Qb + 64;
    const T* Vb = Qb + 128;
    const float scale = 0.125f;   // 1/sqrt(64)
    for (int t = blockIdx.x * 4 + wave; t < tokens; t += gridDim.x * 4) {
        qv[lane] = ld<T>(Qb + (long)t * ldq + lane);
        __builtin_amdgcn_wave_barrier();
        float mx = -INFINITY;
        for (int i = lane; i < tokens; i += 64) {
            const float s = dot64<T>(qv, Kb + (long)i * ldq) * scale;
            sc[i] = s;
            mx = fmaxf(mx, s);
        }
        mx = wave_max(mx);
        float sum = 0.f;
        for (int i = lane; i < tokens; i += 64) {
            const float p = __expf(sc[i] - mx);
            sc[i] = p;
            sum += p;
        }
        sum = wave_sum(sum);
        __builtin_amdgcn_wave_barrier();
        float acc = 0.f;
        for (int i = 0; i < tokens; ++i) acc = fmaf(sc[i], ld<T>(Vb + (long)i * ldq + lane), acc);
        st<T>(o + (row0 + t) * ldo + j * 64 + lane, acc / sum);
        if (lane == 0 && j < n_full) lse[(long)j * rows_total + row0 + t] = mx + __logf(sum);
        __builtin_amdgcn_wave_barrier();
    }
}

// dQ and delta.  grid (row_groups, batch * n_full); dynamic LDS: 4 * (128 + tokens) floats
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const T* __restrict__ qkv, long ldq,
                                                          const T* __restrict__ o, long ldo,
                                                          const float* __restrict__ lse, const T* __restrict__ d_o,
                                                          long ld_do, T* __restrict__ dqkv, long ld_dqkv,
                                                          float* __restrict__ delta, int tokens, int n_full,
                                                          long rows_total) {
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* qv = smem + wave * (128 + tokens);
    float* dov = qv + 64;
    float* sc = dov + 64;
    const int b = blockIdx.y / n_full, j = blockIdx.y % n_full;
    const long row0 = (long)b * tokens;
    const T* Qb = qkv + row0 * ldq + j * 192;
    const T* Kb = Qb + 64;
    const T* Vb = Qb + 128;
    const float scale = 0.125f;
    for (int t = blockIdx.x * 4 + wave; t < tokens; t += gridDim.x * 4) {
        const float dov_l = ld<T>(d_o + (row0 + t) * ld_do + j * 64 + lane);
        qv[lane] = ld<T>(Qb + (long)t * ldq + lane);
        dov[lane] = dov_l;
        const float dl = wave_sum(dov_l * ld<T>(o + (row0 + t) * ldo + j * 64 + lane));
        const float l = lse[(long)j * rows_total + row0 + t];
        __builtin_amdgcn_wave_barrier();
        for (int i = lane; i < tokens; i += 64) {
            const float s = dot64<T>(qv, Kb + (long)i * ldq) * scale;
            const float p = __expf(s - l);
            const float dp = dot64<T>(dov, Vb + (long)i * ldq);
            sc[i] = p * (dp - dl);
        }
        __builtin_amdgcn_wave_barrier();
        float acc = 0.f;
        for (int i = 0; i < tokens; ++i) acc = fmaf(sc[i], ld<T>(Kb + (long)i * ldq + lane), acc);
        st<T>(dqkv + (row0 + t) * ld_dqkv + j * 192 + lane, acc * scale);
        if (lane == 0) delta[(long)j * rows_total + row0 + t] = dl;
        __builtin_amdgcn_wave_barrier();
    }
}

// dK and dV.  One wavefront per key row; lanes first run over query rows, then over channels.
// dynamic LDS: 4 * (128 + 2 * tokens) floats
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const T* __restrict__ qkv, long ldq,
                                                           const float* __restrict__ lse, const T* __restrict__ d_o,
                                                           long ld_do, T* __restrict__ dqkv, long ld_dqkv,
                                                           const float* __restrict__ delta, int tokens, int n_full,
                                                           long rows_total) {
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* kv = smem + wave * (128 + 2 * tokens);
    float* vv = kv + 64;
    float* pb = vv + 64;
    float* dsb = pb + tokens;
    const int b = blockIdx.y / n_full, j = blockIdx.y % n_full;
    const long row0 = (long)b * tokens;
    const T* Qb = qkv + row0 * ldq + j * 192;
    const T* Kb = Qb + 64;
    const T* Vb = Qb + 128;
    const T* dOb = d_o + row0 * ld_do + j * 64;
    const float* lse_b = lse + (long)j * rows_total + row0;
    const float* del_b = delta + (long)j * rows_total + row0;
    const float scale = 0.125f;
    for (int i = blockIdx.x * 4 + wave; i < tokens; i += gridDim.x * 4) {
        kv[lane] = ld<T>(Kb + (long)i * ldq + lane);
        vv[lane] = ld<T>(Vb + (long)i * ldq + lane);
        __builtin_amdgcn_wave_barrier();
        for (int t = lane; t < tokens; t += 64) {
            const float s = dot64<T>(kv, Qb + (long)t * ldq) * scale;
            const float p = __expf(s - lse_b[t]);
            const float dp = dot64<T>(vv, dOb + (long)t * ld_do);
            pb[t] = p;
            dsb[t] = p * (dp - del_b[t]);
        }
        __builtin_amdgcn_wave_barrier();
        float dv = 0.f, dk = 0.f;
        for (int t = 0; t < tokens; ++t) {
            dv = fmaf(pb[t], ld<T>(dOb + (long)t * ld_do + lane), dv);
            dk = fmaf(dsb[t], ld<T>(Qb + (long)t * ldq + lane), dk);
        }
        st<T>(dqkv + (row0 + i) * ld_dqkv + j * 192 + 64 + lane, dk * scale);
        st<T>(dqkv + (row0 + i) * ld_dqkv + j * 192 + 128 + lane, dv);
        __builtin_amdgcn_wave_barrier();
    }
}

static int row_groups(int tokens) {
    int g = (tokens + 3) / 4;
    return g > 16 ? 16 : g;
}

hipError_t launch_attn_fwd_simple(int dtype, const void* qkv, long ldq, void* o, long ldo, float* lse, int batch,
                                  int tokens, int n_live, int n_full, hipStream_t s) {
    if (n_live <= 0) return hipSuccess;
    const dim3 grid(row_groups(tokens), batch * n_live), block(256);
    const size_t lds = sizeof(float) * 4 * (64 + tokens);
    const long rows_total = (long)batch * tokens;
    if (dtype == D2FT_F32)
        hipLaunchKernelGGL(attn_fwd_simple_kernel<float>, grid, block, lds, s, (const float*)qkv, ldq, (float*)o, ldo,
                           lse, tokens, n_live, n_full, rows_total);
    else
        hipLaunchKernelGGL(attn_fwd_simple_kernel<bf16>, grid, block, lds, s, (const bf16*)qkv, ldq, (bf16*)o, ldo,
                           lse, tokens, n_live, n_full, rows_total);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_simple(int dtype, const void* qkv, long ldq, const void* o, long ldo, const float* lse,
                                  const void* d_o, long ld_do, void* dqkv, long ld_dqkv, float* delta, int batch,
                                  int tokens, int n_full, hipStream_t s) {
    if (n_full <= 0) return hipSuccess;
    const dim3 grid(row_groups(tokens), batch * n_full), block(256);
    const long rows_total = (long)batch * tokens;
    const size_t lds1 = sizeof(float) * 4 * (128 + tokens);
    const size_t lds2 = sizeof(float) * 4 * (128 + 2 * tokens);
    if (dtype == D2FT_F32) {
        typedef float T;
        hipLaunchKernelGGL(attn_bwd_dq_kernel<T>, grid, block, lds1, s, (const T*)qkv, ldq, (const T*)o, ldo, lse,
                           (const T*)d_o, ld_do, (T*)dqkv, ld_dqkv, delta, tokens, n_full, rows_total);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_bwd_dkv_kernel<T>, grid, block, lds2, s, (const T*)qkv, ldq, lse, (const T*)d_o, ld_do,
                           (T*)dqkv, ld_dqkv, delta, tokens, n_full, rows_total);
    } else {
        typedef bf16 T;
        hipLaunchKernelGGL(attn_bwd_dq_kernel<T>, grid, block, lds1, s, (const T*)qkv, ldq, (const T*)o, ldo, lse,
                           (const T*)d_o, ld_do, (T*)dqkv, ld_dqkv, delta, tokens, n_full, rows_total);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_bwd_dkv_kernel<T>, grid, block, lds2, s, (const T*)qkv, ldq, lse, (const T*)d_o, ld_do,
                           (T*)dqkv, ld_dqkv, delta, tokens, n_full, rows_total);
    }
    return hipGetLastError();
}

}  // namespace d2ft
