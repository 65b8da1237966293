// General strided GEMM on the vector ALUs with fp32 accumulation.  It is the fp32 path
// (storage type float) and the path for shapes the bf16 MFMA kernel does not take
// (odd strides, tiny or unaligned extents).  64x64 output tile per 256-thread workgroup,
// 4x4 outputs per thread, K staged through LDS 16 at a time.
#include "d2ft_common.h"

namespace d2ft {

constexpr int SG_BM = 64, SG_BN = 64, SG_BK = 16;

template <typename T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmArgs g) {
    __shared__ float As[SG_BK][SG_BM + 4];
    __shared__ float Bs[SG_BK][SG_BN + 4];
    const T* __restrict__ A = static_cast<const T*>(g.A);
    const T* __restrict__ B = static_cast<const T*>(g.B);
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * SG_BM, n0 = blockIdx.x * SG_BN;

    // K range of this split (multiples of SG_BK so that splits do not share a staged slab)
    int kb = 0, ke = g.K;
    if (g.partial) {
        int per = (g.K + g.splits - 1) / g.splits;
        per = (per + SG_BK - 1) / SG_BK * SG_BK;
        kb = blockIdx.z * per;
        ke = min(g.K, kb + per);
    }

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    const bool a_k_contig = (g.a_cs == 1);
    const bool b_k_contig = (g.b_rs == 1);

    for (int k0 = kb; k0 < ke; k0 += SG_BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // A tile: 64 (m) x 16 (k); lanes run along the contiguous index
            int mm, kk;
            if (a_k_contig) {
                kk = tid & 15;
                mm = (tid >> 4) + 16 * i;
            } else {
                mm = tid & 63;
                kk = (tid >> 6) + 4 * i;
            }
            const int m = m0 + mm, k = k0 + kk;
            float v = 0.f;
            if (m < g.M && k < ke) v = ld<T>(A + (long)m * g.a_rs + (long)k * g.a_cs);
            As[kk][mm] = v;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int nn, kk;
            if (b_k_contig) {
                kk = tid & 15;
                nn = (tid >> 4) + 16 * i;
            } else {
                nn = tid & 63;
                kk = (tid >> 6) + 4 * i;
            }
            const int n = n0 + nn, k = k0 + kk;
            float v = 0.f;
            if (n < g.N && k < ke) {
                const int ks = (g.remap == REMAP_B_K) ? g.tbl(k) : k;
                const int ns = (g.remap == REMAP_B_N) ? g.tbl(n) : n;
                v = ld<T>(B + (long)ks * g.b_rs + (long)ns * g.b_cs);
            }
            Bs[kk][nn] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < SG_BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    if (g.partial) {
        float* P = g.partial + (long)blockIdx.z * g.M * g.N;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + ty * 4 + i;
            if (m >= g.M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + tx * 4 + j;
                if (n < g.N) P[(long)m * g.N + n] = acc[i][j];
            }
        }
        return;
    }

    T* __restrict__ C = static_cast<T*>(g.C);
    const T* bias = static_cast<const T*>(g.bias);
    const T* R = static_cast<const T*>(g.residual);
    T* Z = static_cast<T*>(g.Z);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= g.N) continue;
            float v = acc[i][j];
            if (bias) v += ld<T>(bias + (g.bias_remap ? g.tbl(n) : n));
            if (g.act == ACT_GELU) {
                // the activation and its derivative are both taken of the fp32 pre-activation; the
                // derivative is what the backward pass needs, so that is what is saved
                const float zr = v;
                st<T>(Z + (long)m * g.ldz + n, gelu_grad_f(zr));
                v = gelu_f(zr);
            } else if (g.act == ACT_DGELU) {
                v *= ld<T>(Z + (long)m * g.ldz + n);
            }
            if (R) v += ld<T>(R + (long)m * g.ldr + n);
            st<T>(C + (long)m * g.ldc + n, v);
        }
    }
}

hipError_t launch_gemm_simple(const GemmArgs& g, int dtype, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    const int splits = g.partial ? g.splits : 1;
    const dim3 grid((g.N + SG_BN - 1) / SG_BN, (g.M + SG_BM - 1) / SG_BM, splits), block(256);
    if (dtype == D2FT_F32)
        hipLaunchKernelGGL(gemm_simple_kernel<float>, grid, block, 0, s, g);
    else
        hipLaunchKernelGGL(gemm_simple_kernel<bf16>, grid, block, 0, s, g);
    return hipGetLastError();
}

}  // namespace d2ft
