// LayerNorm forward/backward, column sums, split reductions, gradient-slice fills and the
// small LoRA helpers.  All of these are bandwidth-bound: one wavefront owns one row and
// reduces with cross-lane shuffles; column reductions write fp32 partials per row chunk and
// a second kernel sums the partials in a fixed order, so results do not depend on timing.
#include "d2ft_common.h"

namespace d2ft {

// ---------------------------------------------------------------------------
// LayerNorm forward: y = (x - mean) * rstd * gamma + beta, biased variance.
// One wavefront per row; the row is read once and held in registers (NV 8-element vectors per
// lane, width <= 512*NV); NV = 0 is the any-width version that re-reads the row (it then hits L2).
// ---------------------------------------------------------------------------
template <typename T, int NV>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ y,
                                                     float* __restrict__ mean, float* __restrict__ rstd, int rows,
                                                     int width, float eps) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const T* xr = x + (long)row * width;
    T* yr = y + (long)row * width;
    float g[8], b[8], o[8];
    if (NV > 0) {
        float v[NV > 0 ? NV : 1][8];
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            if (c < width) {
                load8(xr + c, v[j]);
#pragma unroll
                for (int i = 0; i < 8; ++i) s += v[j][i];
            }
        }
        const float mu = wave_sum(s) / (float)width;
        float q = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            if (c < width) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float d = v[j][i] - mu;
                    q += d * d;
                }
            }
        }
        const float rs = 1.0f / sqrtf(wave_sum(q) / (float)width + eps);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            if (c < width) {
                load8(gamma + c, g);
                load8(beta + c, b);
#pragma unroll
                for (int i = 0; i < 8; ++i) o[i] = (v[j][i] - mu) * rs * g[i] + b[i];
                store8(yr + c, o);
            }
        }
        if (lane == 0) {
            mean[row] = mu;
            rstd[row] = rs;
        }
    } else {
        float v[8];
        float s = 0.f;
        for (int c = lane * 8; c < width; c += 512) {
            load8(xr + c, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) s += v[i];
        }
        const float mu = wave_sum(s) / (float)width;
        float q = 0.f;
        for (int c = lane * 8; c < width; c += 512) {
            load8(xr + c, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float d = v[i] - mu;
                q += d * d;
            }
        }
        const float rs = 1.0f / sqrtf(wave_sum(q) / (float)width + eps);
        for (int c = lane * 8; c < width; c += 512) {
            load8(xr + c, v);
            load8(gamma + c, g);
            load8(beta + c, b);
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (v[i] - mu) * rs * g[i] + b[i];
            store8(yr + c, o);
        }
        if (lane == 0) {
            mean[row] = mu;
            rstd[row] = rs;
        }
    }
}

// ---------------------------------------------------------------------------
// LayerNorm backward wrt the input, plus a residual: dx = rstd*(dh - mean(dh) - xh*mean(dh*xh)) + res
// Same register caching as the forward kernel (dh and xh are kept).
// ---------------------------------------------------------------------------
template <typename T, int NV>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const T* __restrict__ d, const T* __restrict__ x,
                                                     const float* __restrict__ mean, const float* __restrict__ rstd,
                                                     const T* __restrict__ gamma, const T* res, T* dx, int rows,
                                                     int width) {
    // res and dx may be the same buffer: every lane reads its res elements before it writes them
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const long off = (long)row * width;
    const float mu = mean[row], rs = rstd[row];
    float dv[8], xv[8], g[8], r[8], o[8];
    if (NV > 0) {
        float dh[NV > 0 ? NV : 1][8], xh[NV > 0 ? NV : 1][8];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            if (c < width) {
                load8(d + off + c, dv);
                load8(x + off + c, xv);
                load8(gamma + c, g);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    dh[j][i] = dv[i] * g[i];
                    xh[j][i] = (xv[i] - mu) * rs;
                    s1 += dh[j][i];
                    s2 += dh[j][i] * xh[j][i];
                }
            }
        }
        const float m1 = wave_sum(s1) / (float)width;
        const float m2 = wave_sum(s2) / (float)width;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            if (c < width) {
                if (res) {
                    load8(res + off + c, r);
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) r[i] = 0.f;
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) o[i] = rs * (dh[j][i] - m1 - xh[j][i] * m2) + r[i];
                store8(dx + off + c, o);
            }
        }
    } else {
        float s1 = 0.f, s2 = 0.f;
        for (int c = lane * 8; c < width; c += 512) {
            load8(d + off + c, dv);
            load8(x + off + c, xv);
            load8(gamma + c, g);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float dh = dv[i] * g[i];
                s1 += dh;
                s2 += dh * ((xv[i] - mu) * rs);
            }
        }
        const float m1 = wave_sum(s1) / (float)width;
        const float m2 = wave_sum(s2) / (float)width;
        for (int c = lane * 8; c < width; c += 512) {
            load8(d + off + c, dv);
            load8(x + off + c, xv);
            load8(gamma + c, g);
            if (res) {
                load8(res + off + c, r);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) r[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float xh = (xv[i] - mu) * rs;
                o[i] = rs * (dv[i] * g[i] - m1 - xh * m2) + r[i];
            }
            store8(dx + off + c, o);
        }
    }
}

// ---------------------------------------------------------------------------
// The same backward, also summing columns: of the residual it adds (sum_res) and of the result it
// writes (sum_out) - the gradients of the two biases that sit on the residual stream on either side
// of the feed-forward network.  A workgroup owns kLnSumRows consecutive rows, a wavefront every
// fourth of them; while a wavefront works on one row the loads of its next row are in flight.  The
// wavefront keeps the column sums of its rows in registers, the four wavefronts' sums are added
// through LDS in a fixed order, and the workgroup writes one row of partial sums: [gridDim.x][width].
// ---------------------------------------------------------------------------
constexpr int kLnSumRows = 16;

// 8 consecutive elements as they sit in memory, unpacked to fp32 on use
template <typename T> struct Raw8;
template <> struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float* p) {
        a = *reinterpret_cast<const float4*>(p);
        b = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ __forceinline__ void get(float (&o)[8]) const {
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};
template <> struct Raw8<bf16> {
    uint4 r;
    __device__ __forceinline__ void load(const bf16* p) { r = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void get(float (&o)[8]) const {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

template <typename T, int NV>
__global__ __launch_bounds__(256) void ln_bwd_sums_kernel(const T* __restrict__ d, const T* __restrict__ x,
                                                          const float* __restrict__ mean, const float* __restrict__ rstd,
                                                          const T* __restrict__ gamma, const T* res, T* dx, int rows,
                                                          int width, float* __restrict__ sum_res,
                                                          float* __restrict__ sum_out) {
    __shared__ float red[4][NV * 512];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float sr[NV][8], so[NV][8], g[NV][8];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c = (j * 64 + lane) * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) sr[j][i] = so[j][i] = g[j][i] = 0.f;
        if (c < width) load8(gamma + c, g[j]);
    }
    Raw8<T> nd[NV], nx[NV], nr[NV];   // the next row's d, x, res
    float nmu = 0.f, nrs = 0.f;
    auto fetch = [&](int row) {
        if (row < rows) {
            const long off = (long)row * width;
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const int c = (j * 64 + lane) * 8;
                if (c < width) {
                    nd[j].load(d + off + c);
                    nx[j].load(x + off + c);
                    nr[j].load(res + off + c);
                }
            }
            nmu = mean[row];
            nrs = rstd[row];
        }
    };
    const int row0 = blockIdx.x * kLnSumRows + wave;
    fetch(row0);
#pragma unroll
    for (int it = 0; it < kLnSumRows / 4; ++it) {
        const int row = row0 + it * 4;
        if (row >= rows) break;
        const long off = (long)row * width;
        const float mu = nmu, rs = nrs;
        float dh[NV][8], xh[NV][8], r[NV][8];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            if (c < width) {
                float dv[8], xv[8];
                nd[j].get(dv);
                nx[j].get(xv);
                nr[j].get(r[j]);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    dh[j][i] = dv[i] * g[j][i];
                    xh[j][i] = (xv[i] - mu) * rs;
                    s1 += dh[j][i];
                    s2 += dh[j][i] * xh[j][i];
                }
            }
        }
        if (it + 1 < kLnSumRows / 4) fetch(row + 4);   // in flight under the reductions and the stores below
        const float m1 = wave_sum(s1) / (float)width;
        const float m2 = wave_sum(s2) / (float)width;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            if (c < width) {
                float o[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    o[i] = rs * (dh[j][i] - m1 - xh[j][i] * m2) + r[j][i];
                    sr[j][i] += r[j][i];
                    so[j][i] += o[i];
                }
                store8(dx + off + c, o);
            }
        }
    }
    for (int pass = 0; pass < 2; ++pass) {
        float* out = pass == 0 ? sum_res : sum_out;   // uniform over the grid
        if (!out) continue;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int c = (j * 64 + lane) * 8;
            store8(&red[wave][c], pass == 0 ? sr[j] : so[j]);
        }
        __syncthreads();
        for (int c = threadIdx.x; c < width; c += 256)
            out[(long)blockIdx.x * width + c] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// column sums over a chunk of rows.  A workgroup covers 256 columns (32 lanes x 8 columns, 16-byte
// loads) and 8 row lanes; LN = true sums d*xhat and d (LayerNorm scale / shift gradients).
// ---------------------------------------------------------------------------
template <typename T, bool LN>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ X, long ldx, const T* __restrict__ x,
                                                     const float* __restrict__ mean, const float* __restrict__ rstd,
                                                     int rows, int cols, float* __restrict__ partial,
                                                     float* __restrict__ partial2, int chunks) {
    __shared__ float red[2][8][32][9];
    const int cl = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int col = blockIdx.x * 256 + cl * 8;
    const int per = (rows + chunks - 1) / chunks;
    const int r0 = blockIdx.y * per;
    const int r1 = min(rows, r0 + per);
    float a[8], b[8], dv[8], xv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = b[i] = 0.f;
    if (col < cols) {
        int r = r0 + rg;
        if (!LN) {
            // four rows in flight per thread; each thread still adds its rows in ascending order
            for (; r + 24 < r1; r += 32) {
                float d4[4][8];
#pragma unroll
                for (int j = 0; j < 4; ++j) load8(X + (long)(r + 8 * j) * ldx + col, d4[j]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 8; ++i) a[i] += d4[j][i];
            }
        }
        for (; r < r1; r += 8) {
            load8(X + (long)r * ldx + col, dv);
            if (LN) {
                load8(x + (long)r * ldx + col, xv);
                const float mu = mean[r], rs = rstd[r];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    a[i] += dv[i] * ((xv[i] - mu) * rs);
                    b[i] += dv[i];
                }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) a[i] += dv[i];
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        red[0][rg][cl][i] = a[i];
        if (LN) red[1][rg][cl][i] = b[i];
    }
    __syncthreads();
    // thread t sums column t of the workgroup's 256 over the 8 row lanes, in a fixed order
    const int c2 = threadIdx.x >> 3, i2 = threadIdx.x & 7;
    const int ocol = blockIdx.x * 256 + threadIdx.x;
    if (ocol < cols) {
        float s = 0.f, s2 = 0.f;
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            s += red[0][g][c2][i2];
            if (LN) s2 += red[1][g][c2][i2];
        }
        partial[(long)blockIdx.y * cols + ocol] = s;
        if (LN) partial2[(long)blockIdx.y * cols + ocol] = s2;
    }
}

// ---------------------------------------------------------------------------
// sum split partials in order and write (or add to) the output, with an optional 64-granular remap
// of rows or columns; 4 consecutive columns per thread
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int splits,
                                                              long slice_stride, int rows, int cols,
                                                              T* __restrict__ out, long ldo, int remap,
                                                              int accumulate, Remap64 tbl) {
    const int cq = cols >> 2;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)rows * cq) return;
    const int r = (int)(idx / cq), c = (int)(idx % cq) * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const float* src = partial + (long)r * cols + c;
    // slices are added in index order; eight loads are in flight at a time so that a reduction over many
    // slices is not a chain of memory latencies
    int k = 0;
    for (; k + 8 <= splits; k += 8) {
        float4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = *reinterpret_cast<const float4*>(src + (k + j) * slice_stride);
#pragma unroll
        for (int j = 0; j < 8; ++j) { s.x += v[j].x; s.y += v[j].y; s.z += v[j].z; s.w += v[j].w; }
    }
    for (; k < splits; ++k) {
        const float4 v = *reinterpret_cast<const float4*>(src + k * slice_stride);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    const int ro = (remap == RED_REMAP_ROWS) ? tbl(r) : r;
    const int co = (remap == RED_REMAP_COLS) ? tbl(c) : c;
    T* o = out + (long)ro * ldo + co;
    if (accumulate) {
        s.x += ld<T>(o); s.y += ld<T>(o + 1); s.z += ld<T>(o + 2); s.w += ld<T>(o + 3);
    }
    st<T>(o, s.x); st<T>(o + 1, s.y); st<T>(o + 2, s.z); st<T>(o + 3, s.w);
}

// ---------------------------------------------------------------------------
// Reduction of a grouped weight-gradient launch (see GemmArgs): the splits of tile t left their fp32 partial
// tiles in slots t, t + total_tiles, ...; they are added in split order (eight loads in flight at a time),
// then the sum goes to the tile's place in its problem's output, rows or columns through
// the problem's remap, added to what is there if asked.  blockIdx.y = tile, blockIdx.x = 4 rows of it; a
// thread owns 4 consecutive columns.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void reduce_grouped_kernel(const float* __restrict__ partial, GemmArgs g,
                                                             ReduceGroupedArgs ra, int accumulate) {
    const int t = blockIdx.y;
    int gi = 0;
    while (gi + 1 < g.n_groups && t >= g.grp[gi + 1].tile0) ++gi;
    const GemmGroup G = g.grp[gi];
    const ReduceGroup R = ra.grp[gi];
    const int lt = t - G.tile0;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), c = (threadIdx.x & 63) * 4;
    const int m = (lt % G.tiles_m) * 256 + r, n = (lt / G.tiles_m) * 256 + c;
    if (m >= G.M || n >= G.N) return;
    const float* src = partial + ((long)t * 256 + r) * 256 + c;
    const long stride = (long)g.total_tiles * 256 * 256;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 v[8];   // g.splits <= 8
#pragma unroll
    for (int k = 0; k < 8; ++k)
        if (k < g.splits) v[k] = *reinterpret_cast<const float4*>(src + k * stride);
#pragma unroll
    for (int k = 0; k < 8; ++k)
        if (k < g.splits) { s.x += v[k].x; s.y += v[k].y; s.z += v[k].z; s.w += v[k].w; }
    if (R.remap == RED_REMAP_F32) {
        *reinterpret_cast<float4*>(static_cast<float*>(R.out) + (long)m * R.ldo + n) = s;
        return;
    }
    const int ro = (R.remap == RED_REMAP_ROWS) ? ra.tbl[R.table](m) : m;
    const int co = (R.remap == RED_REMAP_COLS) ? ra.tbl[R.table](n) : n;
    T* o = static_cast<T*>(R.out) + (long)ro * R.ldo + co;
    if (accumulate) {
        s.x += ld<T>(o); s.y += ld<T>(o + 1); s.z += ld<T>(o + 2); s.w += ld<T>(o + 3);
    }
    st<T>(o, s.x); st<T>(o + 1, s.y); st<T>(o + 2, s.z); st<T>(o + 3, s.w);
}

// ---------------------------------------------------------------------------
// up to four column reductions in one launch: blockIdx.y picks the job.  A workgroup owns 32 columns
// (8 threads x 4 columns) and spreads the chunks over 32 row lanes: lane l adds chunks l, l + 32, ... in
// index order (eight loads in flight at a time), then the 32 lanes' sums are added in lane order.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void col_reduce_batch_kernel(ColReduceBatch batch, int accumulate, Remap64 tbl_a,
                                                                Remap64 tbl_b) {
    __shared__ float4 red[32][8];
    const ColReduceJob job = batch.job[blockIdx.y];
    const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
    const int c = blockIdx.x * 32 + cg * 4;
    if (blockIdx.x * 32 >= job.cols) return;   // uniform over the workgroup
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < job.cols) {
        const float* src = job.partial + c;
        int k = rl;
        for (; k + 7 * 32 < job.chunks; k += 8 * 32) {
            float4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = *reinterpret_cast<const float4*>(src + (long)(k + 32 * j) * job.cols);
#pragma unroll
            for (int j = 0; j < 8; ++j) { s.x += v[j].x; s.y += v[j].y; s.z += v[j].z; s.w += v[j].w; }
        }
        for (; k < job.chunks; k += 32) {
            const float4 v = *reinterpret_cast<const float4*>(src + (long)k * job.cols);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    }
    red[rl][cg] = s;
    __syncthreads();
    if (rl != 0 || c >= job.cols) return;
#pragma unroll 8
    for (int l = 1; l < 32; ++l) {
        const float4 v = red[l][cg];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    T* o = static_cast<T*>(job.out) + (job.remap_cols == 1 ? tbl_a(c) : (job.remap_cols == 2 ? tbl_b(c) : c));
    if (accumulate) {
        s.x += ld<T>(o); s.y += ld<T>(o + 1); s.z += ld<T>(o + 2); s.w += ld<T>(o + 3);
    }
    st<T>(o, s.x); st<T>(o + 1, s.y); st<T>(o + 2, s.z); st<T>(o + 3, s.w);
}

// ---------------------------------------------------------------------------
// +0.0 into every gradient slice of the listed heads
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void zero_span(T* base, long count, int tid, int nth) {
    if (!base) return;
    for (long i = tid; i < count; i += nth) base[i] = static_cast<T>(0.0f);
}

template <typename T>
__global__ __launch_bounds__(256) void zero_head_slices_kernel(HeadList heads, int H, int D, int r, T* g_wqkv,
                                                               T* g_bqkv, T* g_wo, T* g_la_q, T* g_la_v, T* g_lb_q,
                                                               T* g_lb_v) {
    const int h = heads.h[blockIdx.y];
    const int tid = blockIdx.x * 256 + threadIdx.x, nth = gridDim.x * 256;
    for (int p = 0; p < 3; ++p) {
        if (g_wqkv) zero_span(g_wqkv + ((long)(p * H + h) * 64) * D, (long)64 * D, tid, nth);
        if (g_bqkv) zero_span(g_bqkv + (long)(p * H + h) * 64, 64, tid, nth);
    }
    if (g_wo) {
        const long hd = (long)H * 64;
        for (long i = tid; i < (long)D * 64; i += nth) g_wo[(i >> 6) * hd + h * 64 + (i & 63)] = static_cast<T>(0.0f);
    }
    if (r > 0) {
        if (g_la_q) zero_span(g_la_q + (long)h * r * D, (long)r * D, tid, nth);
        if (g_la_v) zero_span(g_la_v + (long)h * r * D, (long)r * D, tid, nth);
        if (g_lb_q) zero_span(g_lb_q + (long)h * 64 * r, (long)64 * r, tid, nth);
        if (g_lb_v) zero_span(g_lb_v + (long)h * 64 * r, (long)64 * r, tid, nth);
    }
}

// zero the [tokens][width] block (in x, and in x2 if given) of every (image, position) pair that is
// skipped (which = PAIRS_SKIPPED) or live but not p_f (PAIRS_FORWARD_ONLY) in the image's micro-batch;
// width * sizeof(T) is a multiple of 16 bytes
template <typename T>
__global__ __launch_bounds__(256) void zero_pairs_kernel(T* x, T* x2, long ld, int tokens, int n_pos, int width, int which,
                                                         MicroMask mask) {
    const int b = blockIdx.x / n_pos, p = blockIdx.x % n_pos;
    const int mb = mask.micro_of(b);
    const uint64_t sel = (which == PAIRS_SKIPPED) ? ~mask.live[mb] : (mask.live[mb] & ~mask.full[mb]);
    if (!((sel >> p) & 1)) return;
    constexpr int per = 16 / sizeof(T);
    const int chunks = width / per;
    const long base = (long)b * tokens * ld + (long)p * width;
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = threadIdx.x; i < tokens * chunks; i += 256) {
        const long off = base + (long)(i / chunks) * ld + (i % chunks) * per;
        *reinterpret_cast<float4*>(x + off) = z;
        if (x2) *reinterpret_cast<float4*>(x2 + off) = z;
    }
}

// ---------------------------------------------------------------------------
// +0.0 into the feed-forward gradient slices of the listed heads: rows [h*S, (h+1)*S) of w1 [Dm][D]
// and of b1, columns [h*S, (h+1)*S) of w2 [D][Dm]
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void zero_ffn_slices_kernel(HeadList heads, int S, int D, int Dm, T* g_w1, T* g_b1,
                                                              T* g_w2) {
    const int h = heads.h[blockIdx.y];
    const int tid = blockIdx.x * 256 + threadIdx.x, nth = gridDim.x * 256;
    if (g_w1) zero_span(g_w1 + (long)h * S * D, (long)S * D, tid, nth);
    if (g_b1) zero_span(g_b1 + (long)h * S, S, tid, nth);
    if (g_w2)
        for (long i = tid; i < (long)D * S; i += nth) g_w2[(i / S) * Dm + (long)h * S + (i % S)] = static_cast<T>(0.0f);
}

// ---------------------------------------------------------------------------
// LoRA: effective weights of the compacted heads (Sec. II-D: adapters on query and value)
//   out[(j*3+p)*64 + d][k] = W[p][h][d][k] + scale * sum_i B_p[h][d][i] * A_p[h][i][k],  h = live[j]
// one block per output row
// ---------------------------------------------------------------------------
constexpr int kMaxLoraRank = D2FT_MAX_LORA_RANK;

template <typename T>
__global__ __launch_bounds__(256) void lora_merge_kernel(const T* __restrict__ w_qkv, const T* __restrict__ la_q,
                                                         const T* __restrict__ la_v, const T* __restrict__ lb_q,
                                                         const T* __restrict__ lb_v, T* __restrict__ out,
                                                         HeadList live, int H, int D, int r, float scale) {
    const int row = blockIdx.x;
    const int j = row / 192, p = (row % 192) / 64, d = row % 64;
    const int h = live.h[j];
    const T* wrow = w_qkv + ((long)(p * H + h) * 64 + d) * D;
    const T* A = (p == 0) ? la_q : (p == 2 ? la_v : nullptr);
    const T* B = (p == 0) ? lb_q : (p == 2 ? lb_v : nullptr);
    T* orow = out + (long)row * D;
    __shared__ float bs[kMaxLoraRank + 8];   // this row of B_h, zero padded to a multiple of 8
    if (A) {
        for (int i = threadIdx.x; i < ((r + 7) & ~7); i += 256) bs[i] = i < r ? (float)ld<T>(B + ((long)h * 64 + d) * r + i) : 0.f;
        __syncthreads();
    }
    for (int k = threadIdx.x; k < D; k += 256) {
        float v = ld<T>(wrow + k);
        if (A) {
            float acc = 0.f;
            for (int i0 = 0; i0 < r; i0 += 8) {   // eight rows of A in flight; terms are added in index order
                float a[8];
#pragma unroll
                for (int ii = 0; ii < 8; ++ii) a[ii] = (i0 + ii < r) ? (float)ld<T>(A + ((long)h * r + i0 + ii) * D + k) : 0.f;
#pragma unroll
                for (int ii = 0; ii < 8; ++ii) acc += bs[i0 + ii] * a[ii];
            }
            v += scale * acc;
        }
        st<T>(orow + k, v);
    }
}

// ---------------------------------------------------------------------------
// LoRA gradients from G = gradient of the effective weight (fp32 split partials, rows of head j and
// plane p start at (j*3+p)*64):
//   dA[h][i][k] = scale * sum_d B[h][d][i] * G_h[d][k]      (lora_grad_a_kernel, grid (n_full*2, D/64))
//   dB[h][d][i] = scale * sum_k G_h[d][k] * A[h][i][k]      (lora_grad_b_kernel, grid (n_full*2, 16))
// Each kernel sums the split slices of G itself, in order, and owns complete outputs.
// ---------------------------------------------------------------------------
constexpr int kMaxRank = D2FT_MAX_LORA_RANK;

template <typename T>
__global__ __launch_bounds__(256) void lora_grad_a_kernel(const float* __restrict__ G, int splits, long slice_stride,
                                                          const T* __restrict__ lb_q, const T* __restrict__ lb_v,
                                                          T* g_la_q, T* g_la_v, HeadList full, int D, int r, float scale,
                                                          int accumulate) {
    __shared__ float Bs[64 * kMaxRank];          // B_h [64][r]
    __shared__ float red[4][64];
    const int j = blockIdx.x >> 1, plane = blockIdx.x & 1;
    T* gA = plane == 0 ? g_la_q : g_la_v;
    if (!gA) return;
    const int p = plane == 0 ? 0 : 2;
    const int h = full.h[j];
    const T* B = (plane == 0 ? lb_q : lb_v) + (long)h * 64 * r;
    for (int e = threadIdx.x; e < 64 * r; e += 256) Bs[e] = ld<T>(B + e);
    __syncthreads();
    const int kl = threadIdx.x & 63, dq = threadIdx.x >> 6;   // column within the chunk, group of 16 rows
    const int k = blockIdx.y * 64 + kl;
    // the 16 rows' split slices are added in slice order, 16 loads in flight at a time
    float gs[16];
#pragma unroll
    for (int dd = 0; dd < 16; ++dd) gs[dd] = 0.f;
    if (k < D) {
        const float* src = G + ((long)(j * 3 + p) * 64 + dq * 16) * D + k;
        for (int s = 0; s < splits; ++s) {
#pragma unroll
            for (int dd = 0; dd < 16; ++dd) gs[dd] += src[(long)dd * D + s * slice_stride];
        }
    }
    gA += (long)h * r * D;
    for (int i = 0; i < r; ++i) {
        float acc = 0.f;
#pragma unroll
        for (int dd = 0; dd < 16; ++dd) acc = fmaf(Bs[(dq * 16 + dd) * r + i], gs[dd], acc);
        red[dq][kl] = acc;
        __syncthreads();
        if (dq == 0 && k < D) {
            float v = ((red[0][kl] + red[1][kl]) + (red[2][kl] + red[3][kl])) * scale;
            if (accumulate) v += ld<T>(gA + (long)i * D + k);
            st<T>(gA + (long)i * D + k, v);
        }
        __syncthreads();
    }
}

template <typename T>
__global__ __launch_bounds__(256) void lora_grad_b_kernel(const float* __restrict__ G, int splits, long slice_stride,
                                                          const T* __restrict__ la_q, const T* __restrict__ la_v,
                                                          T* g_lb_q, T* g_lb_v, HeadList full, int D, int r, float scale,
                                                          int accumulate) {
    __shared__ float red[4][4][kMaxRank];        // [wave][row][i]
    const int j = blockIdx.x >> 1, plane = blockIdx.x & 1;
    T* gB = plane == 0 ? g_lb_q : g_lb_v;
    if (!gB) return;
    const int p = plane == 0 ? 0 : 2;
    const int h = full.h[j];
    const T* A = (plane == 0 ? la_q : la_v) + (long)h * r * D;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d0 = blockIdx.y * 4;               // this workgroup's 4 rows of G_h
    // G_h's four rows are summed over the split slices once per group of 16 adapter rows
    for (int i0 = 0; i0 < r; i0 += 16) {
        float acc[4][16];
#pragma unroll
        for (int dd = 0; dd < 4; ++dd)
#pragma unroll
            for (int ii = 0; ii < 16; ++ii) acc[dd][ii] = 0.f;
        for (int k = threadIdx.x; k < D; k += 256) {
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            const float* src = G + ((long)(j * 3 + p) * 64 + d0) * D + k;
            for (int s = 0; s < splits; ++s) {
#pragma unroll
                for (int dd = 0; dd < 4; ++dd) v[dd] += src[(long)dd * D + s * slice_stride];
            }
#pragma unroll
            for (int ii = 0; ii < 16; ++ii) {
                if (i0 + ii < r) {
                    const float a = ld<T>(A + (long)(i0 + ii) * D + k);
#pragma unroll
                    for (int dd = 0; dd < 4; ++dd) acc[dd][ii] = fmaf(v[dd], a, acc[dd][ii]);
                }
            }
        }
#pragma unroll
        for (int ii = 0; ii < 16; ++ii) {
            if (i0 + ii < r) {
#pragma unroll
                for (int dd = 0; dd < 4; ++dd) {
                    const float v = wave_sum(acc[dd][ii]);
                    if (lane == 0) red[wave][dd][i0 + ii] = v;
                }
            }
        }
    }
    __syncthreads();
    gB += (long)h * 64 * r;
    for (int e = threadIdx.x; e < 4 * r; e += 256) {
        const int dd = e / r, i = e % r;
        float v = ((red[0][dd][i] + red[1][dd][i]) + (red[2][dd][i] + red[3][dd][i])) * scale;
        T* o = gB + (long)(d0 + dd) * r + i;
        if (accumulate) v += ld<T>(o);
        st<T>(o, v);
    }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
#define D2FT_DISPATCH(dtype, ...)                  \
    if ((dtype) == D2FT_F32) {                     \
        typedef float T;                           \
        __VA_ARGS__                                \
    } else {                                       \
        typedef bf16 T;                            \
        __VA_ARGS__                                \
    }

// ---------------------------------------------------------------------------
// contribution scores: blockIdx.y = head, blockIdx.x = chunk of one span.  The chunk's threads stride
// over the span in 16-byte (fp32: 32-byte) pieces and add x*x (kind 0) or |x| (kind 1) in fp64; the
// workgroup's 256 sums are added by a fixed tree, the chunks of a head in index order by
// score_final_kernel, so the result does not depend on timing.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void score_partial_kernel(ScoreArgs a, int kind, double* __restrict__ partial) {
    __shared__ double red[256];
    const int h = blockIdx.y, cidx = blockIdx.x;
    int si = 0;
    for (int i = 1; i < a.n; ++i)
        if (cidx >= a.span[i].chunk0) si = i;
    const ScoreSpan sp = a.span[si];
    const T* base = static_cast<const T*>(sp.p) + sp.first + (long)h * sp.head_stride;
    const int n8 = sp.rows * sp.cols8;
    double acc = 0.0;
    for (int i8 = (cidx - sp.chunk0) * 256 + threadIdx.x; i8 < n8; i8 += sp.nchunks * 256) {
        const int r = i8 / sp.cols8, c8 = i8 - r * sp.cols8;
        float v[8];
        load8(base + (long)r * sp.stride + c8 * 8, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const double d = (double)v[j];
            acc += kind == 0 ? d * d : fabs(d);
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[(long)h * a.total_chunks + cidx] = red[0];
}

__global__ void score_final_kernel(const double* __restrict__ partial, int chunks, int H, double* __restrict__ out) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= H) return;
    double s = 0.0;
    for (int c = 0; c < chunks; ++c) s += partial[(long)h * chunks + c];
    out[h] = s;
}

// ---------------------------------------------------------------------------
// SGD with momentum: blockIdx.y = entry of the head list, blockIdx.x = chunk of one span; 8 elements per
// thread and step.  v <- mu*v + (g + wd*w), w <- w - lr*v in fp32; with a master copy the update is
// applied to it and the storage-type weight receives its rounded value.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void sgd_momentum_kernel(SgdArgs a, HeadList heads) {
    const int cidx = blockIdx.x;
    int si = 0;
    for (int i = 1; i < a.n; ++i)
        if (cidx >= a.span[i].chunk0) si = i;
    const SgdSpan sp = a.span[si];
    const long base = sp.first + (long)heads.h[blockIdx.y] * sp.head_stride;
    const int n8 = sp.rows * sp.cols8;
    for (int i8 = (cidx - sp.chunk0) * 256 + threadIdx.x; i8 < n8; i8 += sp.nchunks * 256) {
        const int r = i8 / sp.cols8, c8 = i8 - r * sp.cols8;
        const long off = base + (long)r * sp.stride + c8 * 8;
        float w[8], g[8], v[8];
        T* wp = static_cast<T*>(sp.w) + off;
        if (sp.master) load8(sp.master + off, w); else load8(wp, w);
        load8(static_cast<const T*>(sp.g) + off, g);
        load8(sp.v + off, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[j] = a.momentum * v[j] + (g[j] + a.weight_decay * w[j]);
            w[j] = w[j] - a.lr * v[j];
        }
        store8(sp.v + off, v);
        if (sp.master) store8(sp.master + off, w);
        store8(wp, w);
    }
}

hipError_t launch_ln_fwd(int dtype, const void* x, const void* gamma, const void* beta, void* y, float* mean,
                         float* rstd, int rows, int width, float eps, hipStream_t s) {
    const dim3 grid((rows + 3) / 4), block(256);
#define D2FT_LN_FWD(NV)                                                                                        \
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL((ln_fwd_kernel<T, NV>), grid, block, 0, s, (const T*)x, (const T*)gamma, \
                                            (const T*)beta, (T*)y, mean, rstd, rows, width, eps);)
    if (width <= 512) { D2FT_LN_FWD(1) } else if (width <= 1024) { D2FT_LN_FWD(2) } else if (width <= 2048) { D2FT_LN_FWD(4) } else { D2FT_LN_FWD(0) }
#undef D2FT_LN_FWD
    return hipGetLastError();
}

bool ln_bwd_sums_supported(int width) { return width <= 2048; }
int ln_bwd_sums_bands(int rows) { return (rows + kLnSumRows - 1) / kLnSumRows; }

hipError_t launch_ln_bwd_sums(int dtype, const void* d, const void* x, const float* mean, const float* rstd,
                              const void* gamma, const void* res, void* dx, int rows, int width, float* sum_res,
                              float* sum_out, hipStream_t s) {
    if (!ln_bwd_sums_supported(width) || !res) return hipErrorNotSupported;
    const dim3 grid(ln_bwd_sums_bands(rows)), block(256);
#define D2FT_LN_BWD_SUMS(NV)                                                                                         \
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL((ln_bwd_sums_kernel<T, NV>), grid, block, 0, s, (const T*)d, (const T*)x, \
                                            mean, rstd, (const T*)gamma, (const T*)res, (T*)dx, rows, width, sum_res,  \
                                            sum_out);)
    if (width <= 512) { D2FT_LN_BWD_SUMS(1) } else if (width <= 1024) { D2FT_LN_BWD_SUMS(2) } else { D2FT_LN_BWD_SUMS(4) }
#undef D2FT_LN_BWD_SUMS
    return hipGetLastError();
}

hipError_t launch_ln_bwd(int dtype, const void* d, const void* x, const float* mean, const float* rstd,
                         const void* gamma, const void* res, void* dx, int rows, int width, hipStream_t s) {
    const dim3 grid((rows + 3) / 4), block(256);
#define D2FT_LN_BWD(NV)                                                                                             \
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL((ln_bwd_kernel<T, NV>), grid, block, 0, s, (const T*)d, (const T*)x, mean, \
                                            rstd, (const T*)gamma, (const T*)res, (T*)dx, rows, width);)
    if (width <= 512) { D2FT_LN_BWD(1) } else if (width <= 1024) { D2FT_LN_BWD(2) } else if (width <= 2048) { D2FT_LN_BWD(4) } else { D2FT_LN_BWD(0) }
#undef D2FT_LN_BWD
    return hipGetLastError();
}

hipError_t launch_ln_param_grad(int dtype, const void* d, const void* x, const float* mean, const float* rstd,
                                float* partial_g, float* partial_b, int rows, int width, int chunks, hipStream_t s) {
    const dim3 grid((width + 255) / 256, chunks), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL((colsum_kernel<T, true>), grid, block, 0, s, (const T*)d, (long)width,
                                            (const T*)x, mean, rstd, rows, width, partial_g, partial_b, chunks);)
    return hipGetLastError();
}

hipError_t launch_colsum(int dtype, const void* X, long ld, int rows, int cols, float* partial, int chunks,
                         hipStream_t s) {
    const dim3 grid((cols + 255) / 256, chunks), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL((colsum_kernel<T, false>), grid, block, 0, s, (const T*)X, ld,
                                            (const T*)nullptr, (const float*)nullptr, (const float*)nullptr, rows,
                                            cols, partial, (float*)nullptr, chunks);)
    return hipGetLastError();
}

hipError_t launch_reduce_partials(int dtype, const float* partial, int splits, long slice_stride, int rows, int cols,
                                  void* out, long ldo, int remap, const Remap64& tbl, int accumulate,
                                  hipStream_t s) {
    const long total = (long)rows * (cols / 4);   // cols is a multiple of 8 at every call site
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(reduce_partials_kernel<T>, grid, block, 0, s, partial, splits,
                                            slice_stride, rows, cols, (T*)out, ldo, remap, accumulate, tbl);)
    return hipGetLastError();
}

hipError_t launch_reduce_grouped(int dtype, const GemmArgs& g, const ReduceGroupedArgs& r, int accumulate, hipStream_t s) {
    if (g.total_tiles <= 0) return hipSuccess;
    const dim3 grid(64, g.total_tiles), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(reduce_grouped_kernel<T>, grid, block, 0, s, g.partial, g, r, accumulate);)
    return hipGetLastError();
}

hipError_t launch_subnet_scores(int dtype, const ScoreArgs& a, int kind, double* partial, double* out, hipStream_t s) {
    const dim3 grid(a.total_chunks, a.H), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(score_partial_kernel<T>, grid, block, 0, s, a, kind, partial);)
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(score_final_kernel, dim3((a.H + 63) / 64), dim3(64), 0, s, partial, a.total_chunks, a.H, out);
    return hipGetLastError();
}

hipError_t launch_sgd(int dtype, const SgdArgs& a, const HeadList& heads, hipStream_t s) {
    if (a.n <= 0 || heads.n <= 0) return hipSuccess;
    const dim3 grid(a.total_chunks, heads.n), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(sgd_momentum_kernel<T>, grid, block, 0, s, a, heads);)
    return hipGetLastError();
}

hipError_t launch_col_reduce_batch(int dtype, const ColReduceBatch& batch, const Remap64& tbl_a, const Remap64& tbl_b,
                                   int accumulate, hipStream_t s) {
    if (batch.n <= 0) return hipSuccess;
    int cols = 0;
    for (int i = 0; i < batch.n; ++i) cols = batch.job[i].cols > cols ? batch.job[i].cols : cols;   // multiples of 8
    const dim3 grid((unsigned)((cols + 31) / 32), batch.n), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(col_reduce_batch_kernel<T>, grid, block, 0, s, batch, accumulate, tbl_a, tbl_b);)
    return hipGetLastError();
}

hipError_t launch_zero_ffn_slices(int dtype, const HeadList& heads, int slice, int D, int Dm, void* g_w1, void* g_b1,
                                  void* g_w2, hipStream_t s) {
    if (heads.n <= 0 || (!g_w1 && !g_b1 && !g_w2)) return hipSuccess;
    const dim3 grid(32, heads.n), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(zero_ffn_slices_kernel<T>, grid, block, 0, s, heads, slice, D, Dm, (T*)g_w1,
                                            (T*)g_b1, (T*)g_w2);)
    return hipGetLastError();
}

hipError_t launch_zero_pairs(int dtype, void* x, void* x2, long ld, int batch, int tokens, int n_pos, int width, int which,
                             const MicroMask& mask, hipStream_t s) {
    if (n_pos <= 0 || batch <= 0) return hipSuccess;
    const dim3 grid(batch * n_pos), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(zero_pairs_kernel<T>, grid, block, 0, s, (T*)x, (T*)x2, ld, tokens, n_pos, width,
                                            which, mask);)
    return hipGetLastError();
}

hipError_t launch_zero_head_slices(int dtype, const HeadList& heads, int H, int D, int r, void* g_wqkv, void* g_bqkv,
                                   void* g_wo, void* g_la_q, void* g_la_v, void* g_lb_q, void* g_lb_v,
                                   hipStream_t s) {
    if (heads.n <= 0) return hipSuccess;
    const dim3 grid(32, heads.n), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(zero_head_slices_kernel<T>, grid, block, 0, s, heads, H, D, r,
                                            (T*)g_wqkv, (T*)g_bqkv, (T*)g_wo, (T*)g_la_q, (T*)g_la_v, (T*)g_lb_q,
                                            (T*)g_lb_v);)
    return hipGetLastError();
}

hipError_t launch_lora_merge(int dtype, const void* w_qkv, const void* la_q, const void* la_v, const void* lb_q,
                             const void* lb_v, void* out, const HeadList& live, int n_heads_used, int H, int D, int r,
                             float scale, hipStream_t s) {
    if (n_heads_used <= 0) return hipSuccess;
    const dim3 grid(n_heads_used * 192), block(256);
    D2FT_DISPATCH(dtype, hipLaunchKernelGGL(lora_merge_kernel<T>, grid, block, 0, s, (const T*)w_qkv, (const T*)la_q,
                                            (const T*)la_v, (const T*)lb_q, (const T*)lb_v, (T*)out, live, H, D, r,
                                            scale);)
    return hipGetLastError();
}

hipError_t launch_lora_project(int dtype, const float* G, int splits, long slice_stride, const void* la_q,
                               const void* la_v, const void* lb_q, const void* lb_v, void* g_la_q, void* g_la_v,
                               void* g_lb_q, void* g_lb_v, const HeadList& full, int H, int D, int r, float scale,
                               int accumulate, hipStream_t s) {
    (void)H;
    if (full.n <= 0) return hipSuccess;
    const dim3 block(256);
    if (g_la_q || g_la_v) {
        const dim3 grid(full.n * 2, (D + 63) / 64);
        D2FT_DISPATCH(dtype, hipLaunchKernelGGL(lora_grad_a_kernel<T>, grid, block, 0, s, G, splits, slice_stride,
                                                (const T*)lb_q, (const T*)lb_v, (T*)g_la_q, (T*)g_la_v, full, D, r, scale,
                                                accumulate);)
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (g_lb_q || g_lb_v) {
        const dim3 grid(full.n * 2, 16);
        D2FT_DISPATCH(dtype, hipLaunchKernelGGL(lora_grad_b_kernel<T>, grid, block, 0, s, G, splits, slice_stride,
                                                (const T*)la_q, (const T*)la_v, (T*)g_lb_q, (T*)g_lb_v, full, D, r, scale,
                                                accumulate);)
    }
    return hipGetLastError();
}

}  // namespace d2ft
