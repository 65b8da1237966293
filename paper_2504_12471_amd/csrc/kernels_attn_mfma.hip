// Fused softmax attention on the CDNA4 matrix cores for head dimension 64 and up to 256 tokens
// (bf16 storage, fp32 accumulate).  One 256-thread workgroup owns one (image, head); K and V of
// that pair stay in LDS for the whole kernel.
//
// Everything is computed in the transposed orientation S^T = K Q^T so that, in the MFMA result
// layout, one lane owns ONE query column: the row-wise softmax reductions are then in-lane plus a
// single cross-lane exchange, and a lane's 8 consecutive accumulator elements are exactly the
// 8 k-slots the next MFMA wants, so probabilities go from the S^T accumulators into the P.V
// product without leaving registers.  Operands whose reduction index is not their contiguous
// index (V in the forward pass; Q, K, dO in the backward pass) are read from their natural
// [token][channel] layout with the transposing LDS load (ds_read_b64_tr_b16).
//
// MFMA 32x32x16 bf16 layouts used throughout (h = lane / 32, c = lane % 32):
//   operand:  row-or-column c, k-slots 8h .. 8h+7
//   result :  column c, element e <-> row 8*(e/4) + 4h + e%4
#include <type_traits>

#include "d2ft_common.h"

namespace d2ft {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

namespace {

constexpr float kScale = 0.125f;                         // 1/sqrt(64)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int e = 0; e < 16; ++e) z[e] = 0.f;
    return z;
}

// row-form operand: 8 consecutive channels of row `row` starting at channel ch (16-byte LDS read)
__device__ __forceinline__ bf16x8 frag_rows(const bf16* lds, int stride, int row, int ch) {
    return *reinterpret_cast<const bf16x8*>(lds + row * stride + ch);
}

// transposed operand from a [token][channel] tile: the lane gets, for channel ch0 + c, the tokens
// t0 + 4h + {0..3} (slots 0..3) and t0 + 8 + 4h + {0..3} (slots 4..7): the slot order in which a lane
// holds 8 consecutive result elements of a transposed score tile.
__device__ __forceinline__ bf16x8 frag_tr(const bf16* lds, int stride, int t0, int ch0, int lane) {
    const int j = lane & 15;
    const bf16* p = lds + (t0 + 4 * (lane >> 5) + (j >> 2)) * stride + ch0 + 16 * ((lane >> 4) & 1) + 4 * (j & 3);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 8 * stride));
    s16x8 r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return __builtin_bit_cast(bf16x8, r);
}

// 8 consecutive result elements -> bf16 operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = static_cast<__bf16>(v[first + i]);
    return r;
}

// copy rows [0, rows_valid) x 64 channels of a [token][ld] global tile to LDS rows of `stride`, zero rows above.
// All global loads of the tile are issued before the first LDS store, so their latencies overlap.
template <int TP>
__device__ __forceinline__ void load_tile64(const bf16* __restrict__ g, long ld, int rows_valid, bf16* lds, int stride) {
    constexpr int N = TP * 8 / 256;
    u32x4 v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = threadIdx.x + i * 256;
        const int r = c >> 3, ch = (c & 7) * 8;
        v[i] = u32x4{0u, 0u, 0u, 0u};
        if (r < rows_valid) v[i] = *reinterpret_cast<const u32x4*>(g + (long)r * ld + ch);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = threadIdx.x + i * 256;
        *reinterpret_cast<u32x4*>(lds + (c >> 3) * stride + (c & 7) * 8) = v[i];
    }
}
// the same for two tiles at once (K and V): twice the loads in flight
template <int TP, int NTHR = 256>
__device__ __forceinline__ void load_two_tiles64(const bf16* __restrict__ g0, const bf16* __restrict__ g1, long ld,
                                                 int rows_valid, bf16* lds0, int stride0, bf16* lds1, int stride1) {
    constexpr int N = (TP * 8 + NTHR - 1) / NTHR;
    u32x4 v0[N], v1[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = threadIdx.x + i * NTHR;
        const int r = c >> 3, ch = (c & 7) * 8;
        v0[i] = u32x4{0u, 0u, 0u, 0u};
        v1[i] = u32x4{0u, 0u, 0u, 0u};
        if (r < rows_valid) {   // rows_valid <= TP, so chunks past the tile are skipped as well
            v0[i] = *reinterpret_cast<const u32x4*>(g0 + (long)r * ld + ch);
            v1[i] = *reinterpret_cast<const u32x4*>(g1 + (long)r * ld + ch);
        }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = threadIdx.x + i * NTHR;
        if (TP * 8 % NTHR == 0 || c < TP * 8) {
            *reinterpret_cast<u32x4*>(lds0 + (c >> 3) * stride0 + (c & 7) * 8) = v0[i];
            *reinterpret_cast<u32x4*>(lds1 + (c >> 3) * stride1 + (c & 7) * 8) = v1[i];
        }
    }
}

constexpr int kKS = 72;   // K rows in LDS: 144 bytes (row-form reads)
constexpr int kVS = 96;   // V rows in LDS: 192 bytes (transposing reads)

// ---------------------------------------------------------------------------
// forward: O = softmax(Q K^T / 8) V per (image, live head); log-sum-exp saved for p_f heads
// ---------------------------------------------------------------------------
struct WholeBatch {};   // no mask: every (image, head) pair is live, the first n_full positions are p_f

template <int KT, typename Mask>   // KT: number of 32-token tiles
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv, long ldq,
                                                            bf16* __restrict__ o, long ldo, float* __restrict__ lse,
                                                            int tokens, int n_live, int n_full, long rows_total,
                                                            Mask mask) {
    constexpr int TP = KT * 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* Ks = reinterpret_cast<bf16*>(smem_raw);
    bf16* Vs = Ks + TP * kKS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int b = blockIdx.x / n_live;   // with a mask n_live is the number of slots per image
    int j = blockIdx.x % n_live;
    const long row0 = (long)b * tokens;
    bool save_lse = j < n_full;
    if constexpr (std::is_same<Mask, MicroMask>::value) {
        const int mb = mask.micro_of(b), slot = j;
        const uint64_t live = mask.live[mb];
        const uint64_t skipped = ~live & (mask.n_live_pos >= 64 ? ~0ull : ((1ull << mask.n_live_pos) - 1ull));
        int r = 0;
        for (uint64_t m = skipped; m; m &= m - 1, ++r)   // heads skipped in this image's micro-batch: O = 0
            if (r % n_live == slot) {
                const int p = __builtin_ctzll(m);
                const u32x4 z = {0u, 0u, 0u, 0u};
                for (int i = threadIdx.x; i < tokens * 8; i += 256)
                    *reinterpret_cast<u32x4*>(o + (row0 + (i >> 3)) * ldo + p * 64 + (i & 7) * 8) = z;
            }
        if (slot >= __builtin_popcountll(live)) return;
        uint64_t m = live;
        for (int t = 0; t < slot; ++t) m &= m - 1;
        j = __builtin_ctzll(m);   // this slot's live head
        save_lse = (mask.full[mb] >> j) & 1;
    }
    const bf16* Qb = qkv + row0 * ldq + j * 192;
    load_two_tiles64<TP>(Qb + 64, Qb + 128, ldq, tokens, Ks, kKS, Vs, kVS);
    __syncthreads();

    for (int qt = wave; qt < KT; qt += 4) {
        const int q = qt * 32 + c;
        const bool q_ok = q < tokens;
        bf16x8 qf[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (q_ok) v = *reinterpret_cast<const u32x4*>(Qb + (long)q * ldq + kk * 16 + 8 * h);
            qf[kk] = __builtin_bit_cast(bf16x8, v);
        }
        // S^T tiles: rows = keys of tile u, column = this lane's query.  K fragments of tile u+1 are
        // fetched from LDS while the MFMAs of tile u run (one read behind each MFMA).
        f32x16 s[KT];
        const f32x16 zero_acc = zero16();   // shared C operand of every tile's first MFMA
        bf16x8 kf[2][4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kf[0][kk] = frag_rows(Ks, kKS, c, kk * 16 + 8 * h);
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            if (u + 1 < KT) {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) kf[(u + 1) & 1][kk] = frag_rows(Ks, kKS, (u + 1) * 32 + c, kk * 16 + 8 * h);
            }
            s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[u & 1][0], qf[0], zero_acc, 0, 0, 0);
#pragma unroll
            for (int kk = 1; kk < 4; ++kk)
                s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[u & 1][kk], qf[kk], s[u], 0, 0, 0);
            if (u + 1 < KT) {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // first V fragments are fetched under the softmax arithmetic
        bf16x8 vf[2][4];
#pragma unroll
        for (int gp = 0; gp < 2; ++gp)
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) vf[0][gp * 2 + dt] = frag_tr(Vs, kVS, 16 * gp, dt * 32, lane);
        float m = -INFINITY;
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            if (u * 32 + 31 >= tokens) {   // only tiles that reach past the last token need the mask
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = u * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                    if (key >= tokens) s[u][e] = -INFINITY;
                }
            }
            // three-input maxima: half the instructions of a chain of two-input ones
            float t0 = fmaxf(fmaxf(s[u][0], s[u][1]), s[u][2]);
            float t1 = fmaxf(fmaxf(s[u][3], s[u][4]), s[u][5]);
            float t2 = fmaxf(fmaxf(s[u][6], s[u][7]), s[u][8]);
            float t3 = fmaxf(fmaxf(s[u][9], s[u][10]), s[u][11]);
            float t4 = fmaxf(fmaxf(s[u][12], s[u][13]), s[u][14]);
            t0 = fmaxf(fmaxf(t0, t1), t2);
            t3 = fmaxf(fmaxf(t3, t4), s[u][15]);
            m = fmaxf(fmaxf(m, t0), t3);
        }
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        const float cexp = kScale * kLog2e;
        const float mc = m * cexp;
        float sum = 0.f;
#pragma unroll
        for (int u = 0; u < KT; ++u)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[u][e], cexp, -mc));
                s[u][e] = p;
                sum += p;
            }
        sum += __shfl_xor(sum, 32, 64);
        // O^T = V^T P^T: rows = channels, column = this lane's query; V fragments one tile ahead
        f32x16 ot[2] = {zero16(), zero16()};
#pragma unroll
        for (int u = 0; u < KT; ++u) {
            if (u + 1 < KT) {
#pragma unroll
                for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
                        vf[(u + 1) & 1][gp * 2 + dt] = frag_tr(Vs, kVS, (u + 1) * 32 + 16 * gp, dt * 32, lane);
            }
#pragma unroll
            for (int gp = 0; gp < 2; ++gp) {
                const bf16x8 pf = pack8(s[u], 8 * gp);
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
                    ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u & 1][gp * 2 + dt], pf, ot[dt], 0, 0, 0);
            }
            if (u + 1 < KT) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (q_ok) {
            const float inv = 1.0f / sum;
            bf16* orow = o + (row0 + q) * ldo + j * 64;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    uint2 pk;
                    pk.x = pack_bf16x2(ot[dt][4 * eg] * inv, ot[dt][4 * eg + 1] * inv);
                    pk.y = pack_bf16x2(ot[dt][4 * eg + 2] * inv, ot[dt][4 * eg + 3] * inv);
                    *reinterpret_cast<uint2*>(orow + dt * 32 + 8 * eg + 4 * h) = pk;
                }
            if (h == 0 && save_lse) lse[(long)j * rows_total + row0 + q] = m * kScale + __logf(sum);
        }
    }
}

template <int KT, typename Mask>
hipError_t launch_fwd_kt(const bf16* qkv, long ldq, bf16* o, long ldo, float* lse, int batch, int tokens, int n_live,
                         int n_full, const Mask& mask, hipStream_t s) {
    constexpr size_t lds = (size_t)KT * 32 * (kKS + kVS) * sizeof(bf16);
    auto kern = attn_fwd_mfma_kernel<KT, Mask>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(batch * n_live), dim3(256), lds, s, qkv, ldq, o, ldo, lse, tokens, n_live, n_full,
                       (long)batch * tokens, mask);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// backward for p_f heads: dQ, dK, dV from Q, K, V, O, dO and the saved log-sum-exp
//
// Per 32x32 tile pair (query tile i, key tile u), in the orientation S = Q K^T (a lane owns one KEY
// column, its 16 result elements are 16 queries):
//     S  = Q_i K_u^T              P  = exp(S/8 - lse_q)          (probabilities are rebuilt, never stored)
//     dP = dO_i V_u^T             dS = P * (dP - delta_q),       delta_q = sum_d dO[q][d] O[q][d]
//     dV_u^T += dO_i^T P          dK_u^T += Q_i^T dS             (P, dS feed the MFMA straight from registers)
//     dQ_i^T += K_u^T dS^T        (dS goes through a 2 KB per-wavefront LDS tile to change owner)
// The workgroup has eight wavefronts; wavefront w owns key tile w (a wavefront beyond the last tile
// only takes part in the loads and barriers) and keeps its dK, dV accumulators in registers for the
// whole kernel.  The partial dQ_i tiles are summed through four LDS slots in a fixed order:
// wavefronts 0..3 write, wavefronts 4..7 add theirs onto slot w-4, then the slots are added as
// (0+1)+(2+3).
// ---------------------------------------------------------------------------
constexpr int kTS = 104;   // rows that are read both ways (row-form and transposing): 208 bytes
constexpr int kBwdWaves = 8;

template <int KT, typename Mask>
__global__ __launch_bounds__(64 * kBwdWaves, 2) void attn_bwd_mfma_kernel(const bf16* __restrict__ qkv, long ldq,
                                                                          const bf16* __restrict__ o, long ldo,
                                                                          const float* __restrict__ lse,
                                                                          const bf16* __restrict__ d_o, long ld_do,
                                                                          bf16* __restrict__ dqkv, long ld_dqkv,
                                                                          int tokens, int n_full, long rows_total,
                                                                          Mask mask) {
    static_assert(KT <= kBwdWaves, "one key tile per wavefront");
    constexpr int TP = KT * 32;
    constexpr int NTHR = 64 * kBwdWaves;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* Ks = reinterpret_cast<bf16*>(smem_raw);        // [TP][kTS]
    bf16* Vs = Ks + TP * kTS;                            // [TP][kKS]
    bf16* Qs = Vs + TP * kKS;                            // [32][kTS]   current query tile
    bf16* dOs = Qs + 32 * kTS;                           // [32][kTS]
    bf16* dSs_all = dOs + 32 * kTS;                      // [8][32 keys][32 queries]
    float* lse_s = reinterpret_cast<float*>(dSs_all + kBwdWaves * 32 * 32);   // [TP]
    float* del_s = lse_s + TP;                           // [TP]
    float* dQp = del_s + TP;                             // [4][64 channels][32 queries]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    bf16* dSs = dSs_all + wave * 32 * 32;
    const int b = blockIdx.x / n_full;   // with a mask n_full is the number of slots per image
    int j = blockIdx.x % n_full;
    const long row0 = (long)b * tokens;
    if constexpr (std::is_same<Mask, MicroMask>::value) {
        const int mb = mask.micro_of(b), slot = j;
        const uint64_t full = mask.full[mb];
        const uint64_t rest = ~full & (mask.n_full_pos >= 64 ? ~0ull : ((1ull << mask.n_full_pos) - 1ull));
        int r = 0;
        for (uint64_t m = rest; m; m &= m - 1, ++r)   // not p_f in this image's micro-batch: dQ = dK = dV = 0
            if (r % n_full == slot) {
                bf16* zb = dqkv + row0 * ld_dqkv + __builtin_ctzll(m) * 192;
                const u32x4 z = {0u, 0u, 0u, 0u};
                for (int i = threadIdx.x; i < tokens * 24; i += NTHR)
                    *reinterpret_cast<u32x4*>(zb + (long)(i / 24) * ld_dqkv + (i % 24) * 8) = z;
            }
        if (slot >= __builtin_popcountll(full)) return;
        uint64_t m = full;
        for (int t = 0; t < slot; ++t) m &= m - 1;
        j = __builtin_ctzll(m);   // this slot's p_f head
    }
    const bf16* Qb = qkv + row0 * ldq + j * 192;
    const bf16* dOb = d_o + row0 * ld_do + j * 64;
    const bf16* Ob = o + row0 * ldo + j * 64;
    bf16* dQb = dqkv + row0 * ld_dqkv + j * 192;

    load_two_tiles64<TP, NTHR>(Qb + 64, Qb + 128, ldq, tokens, Ks, kTS, Vs, kKS);
    for (int q = threadIdx.x; q < TP; q += NTHR) {
        float l = 0.f, dl = 0.f;
        if (q < tokens) {
            l = lse[(long)j * rows_total + row0 + q];
            u32x4 a[8], g[8];
#pragma unroll
            for (int ch = 0; ch < 8; ++ch) {
                a[ch] = *reinterpret_cast<const u32x4*>(dOb + (long)q * ld_do + ch * 8);
                g[ch] = *reinterpret_cast<const u32x4*>(Ob + (long)q * ldo + ch * 8);
            }
#pragma unroll
            for (int ch = 0; ch < 8; ++ch)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    dl = fmaf(__uint_as_float(a[ch][i] << 16), __uint_as_float(g[ch][i] << 16), dl);
                    dl = fmaf(__uint_as_float(a[ch][i] & 0xffff0000u), __uint_as_float(g[ch][i] & 0xffff0000u), dl);
                }
        }
        lse_s[q] = l * kLog2e;
        del_s[q] = dl;
    }

    const int u = wave;                 // this wavefront's key tile
    const bool has_tile = u < KT;
    f32x16 dKt[2], dVt[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
        dKt[dt] = zero16();
        dVt[dt] = zero16();
    }
    const float cexp = kScale * kLog2e;

    // one 16-byte chunk of Q_i (threads 0..255) or of dO_i (threads 256..511) per thread; the chunks of
    // tile i+1 are fetched while tile i is processed
    const int ld_t = threadIdx.x & 255;
    const int ld_r = ld_t >> 3, ld_ch = (ld_t & 7) * 8;
    const bool ld_q = threadIdx.x < 256;
    const bf16* ld_src = ld_q ? Qb : dOb;
    const long ld_ld = ld_q ? ldq : ld_do;
    bf16* ld_dst = (ld_q ? Qs : dOs) + ld_r * kTS + ld_ch;
    u32x4 nx = {0u, 0u, 0u, 0u};
    if (ld_r < tokens) nx = *reinterpret_cast<const u32x4*>(ld_src + (long)ld_r * ld_ld + ld_ch);
    for (int i = 0; i < KT; ++i) {
        __syncthreads();   // previous query tile fully consumed (and the prologue's LDS writes are visible)
        *reinterpret_cast<u32x4*>(ld_dst) = nx;
        {
            const int q = (i + 1) * 32 + ld_r;
            nx = u32x4{0u, 0u, 0u, 0u};
            if (i + 1 < KT && q < tokens) nx = *reinterpret_cast<const u32x4*>(ld_src + (long)q * ld_ld + ld_ch);
        }
        __syncthreads();
        f32x16 dqt[2] = {zero16(), zero16()};
        if (has_tile) {
            float L[16], DL[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int ql = i * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
                L[e] = lse_s[ql];
                DL[e] = del_s[ql];
            }
            f32x16 s = zero16(), dp = zero16();
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Qs, kTS, c, kk * 16 + 8 * h),
                                                            frag_rows(Ks, kTS, u * 32 + c, kk * 16 + 8 * h), s, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(dOs, kTS, c, kk * 16 + 8 * h),
                                                             frag_rows(Vs, kKS, u * 32 + c, kk * 16 + 8 * h), dp, 0, 0, 0);
            }
            const bool key_ok = (u * 32 + c) < tokens;
            f32x16 ds;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = key_ok ? __builtin_amdgcn_exp2f(s[e] * cexp - L[e]) : 0.f;
                s[e] = p;
                ds[e] = p * (dp[e] - DL[e]);
            }
            // hand dS to the lanes that own queries: [key][query] tile, 8-byte writes
#pragma unroll
            for (int eg = 0; eg < 4; ++eg) {
                uint2 pk;
                pk.x = pack_bf16x2(ds[4 * eg], ds[4 * eg + 1]);
                pk.y = pack_bf16x2(ds[4 * eg + 2], ds[4 * eg + 3]);
                *reinterpret_cast<uint2*>(dSs + c * 32 + 8 * eg + 4 * h) = pk;
            }
#pragma unroll
            for (int gp = 0; gp < 2; ++gp) {
                const bf16x8 pf = pack8(s, 8 * gp);
                const bf16x8 dsf = pack8(ds, 8 * gp);
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    dVt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(dOs, kTS, 16 * gp, dt * 32, lane), pf,
                                                                      dVt[dt], 0, 0, 0);
                    dKt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(Qs, kTS, 16 * gp, dt * 32, lane), dsf,
                                                                      dKt[dt], 0, 0, 0);
                }
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int gp = 0; gp < 2; ++gp) {
                const bf16x8 dst = frag_tr(dSs, 32, 16 * gp, 0, lane);   // column = query c, slots = keys
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
                    dqt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(Ks, kTS, u * 32 + 16 * gp, dt * 32, lane), dst,
                                                                      dqt[dt], 0, 0, 0);
            }
        }
        // partial dQ_i^T of this wavefront: rows = channels, column = query c
        float* slot = dQp + (wave & 3) * 64 * 32;
        if (wave < 4) {
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) slot[(dt * 32 + 8 * (e >> 2) + 4 * h + (e & 3)) * 32 + c] = dqt[dt][e];
        }
        __syncthreads();
        if (wave >= 4 && has_tile) {
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) slot[(dt * 32 + 8 * (e >> 2) + 4 * h + (e & 3)) * 32 + c] += dqt[dt][e];
        }
        __syncthreads();
        {
            const int q = threadIdx.x & 31, dch = threadIdx.x >> 5;   // 16 groups of 4 channels
            float v[4];
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int d = dch * 4 + i4;
                v[i4] = ((dQp[(0 * 64 + d) * 32 + q] + dQp[(1 * 64 + d) * 32 + q]) +
                         (dQp[(2 * 64 + d) * 32 + q] + dQp[(3 * 64 + d) * 32 + q])) * kScale;
            }
            const int qg = i * 32 + q;
            if (qg < tokens) {
                uint2 pk;
                pk.x = pack_bf16x2(v[0], v[1]);
                pk.y = pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<uint2*>(dQb + (long)qg * ld_dqkv + dch * 4) = pk;
            }
        }
    }

    // dK^T, dV^T: rows = channels, column = key owned by the lane -> 8-byte stores of 4 channels
    {
        const int key = u * 32 + c;
        if (has_tile && key < tokens) {
            bf16* krow = dQb + (long)key * ld_dqkv + 64;
            bf16* vrow = krow + 64;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    const int d = dt * 32 + 8 * eg + 4 * h;
                    uint2 pk;
                    pk.x = pack_bf16x2(dKt[dt][4 * eg] * kScale, dKt[dt][4 * eg + 1] * kScale);
                    pk.y = pack_bf16x2(dKt[dt][4 * eg + 2] * kScale, dKt[dt][4 * eg + 3] * kScale);
                    *reinterpret_cast<uint2*>(krow + d) = pk;
                    pk.x = pack_bf16x2(dVt[dt][4 * eg], dVt[dt][4 * eg + 1]);
                    pk.y = pack_bf16x2(dVt[dt][4 * eg + 2], dVt[dt][4 * eg + 3]);
                    *reinterpret_cast<uint2*>(vrow + d) = pk;
                }
        }
    }
}

template <int KT, typename Mask>
hipError_t launch_bwd_kt(const bf16* qkv, long ldq, const bf16* o, long ldo, const float* lse, const bf16* d_o, long ld_do,
                         bf16* dqkv, long ld_dqkv, int batch, int tokens, int n_full, const Mask& mask, hipStream_t s) {
    constexpr int TP = KT * 32;
    constexpr size_t lds = (size_t)(TP * kTS + TP * kKS + 2 * 32 * kTS + kBwdWaves * 32 * 32) * sizeof(bf16) +
                           (size_t)(2 * TP + 4 * 64 * 32) * sizeof(float);
    auto kern = attn_bwd_mfma_kernel<KT, Mask>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(batch * n_full), dim3(64 * kBwdWaves), lds, s, qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv,
                       ld_dqkv, tokens, n_full, (long)batch * tokens, mask);
    return hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(int tokens, long ldq, long ldo) {
    return tokens >= 1 && tokens <= 256 && (ldq % 8) == 0 && (ldo % 8) == 0;
}

template <typename Mask>
static hipError_t attn_fwd_dispatch(const void* qkv, long ldq, void* o, long ldo, float* lse, int batch, int tokens,
                                    int n_live, int n_full, const Mask& mask, hipStream_t s) {
    if (n_live <= 0) return hipSuccess;
    const bf16* q = static_cast<const bf16*>(qkv);
    bf16* op = static_cast<bf16*>(o);
#define D2FT_FWD_CASE(KT) \
    case KT: return launch_fwd_kt<KT, Mask>(q, ldq, op, ldo, lse, batch, tokens, n_live, n_full, mask, s);
    switch ((tokens + 31) / 32) {
        D2FT_FWD_CASE(1) D2FT_FWD_CASE(2) D2FT_FWD_CASE(3) D2FT_FWD_CASE(4)
        D2FT_FWD_CASE(5) D2FT_FWD_CASE(6) D2FT_FWD_CASE(7) D2FT_FWD_CASE(8)
        default: return hipErrorNotSupported;
    }
#undef D2FT_FWD_CASE
}

hipError_t launch_attn_fwd_mfma(const void* qkv, long ldq, void* o, long ldo, float* lse, int batch, int tokens,
                                int n_live, int n_full, hipStream_t s) {
    return attn_fwd_dispatch(qkv, ldq, o, ldo, lse, batch, tokens, n_live, n_full, WholeBatch{}, s);
}

static int busiest(const uint64_t* sel, int n) {   // most pairs that take part in one micro-batch
    int slots = 0;
    for (int i = 0; i < n; ++i) {
        const int c = __builtin_popcountll(sel[i]);
        slots = c > slots ? c : slots;
    }
    return slots;
}

hipError_t launch_attn_fwd_mfma_masked(const void* qkv, long ldq, void* o, long ldo, float* lse, int batch, int tokens,
                                       int n_live, const MicroMask& mask, hipStream_t s) {
    if (n_live != mask.n_live_pos) return hipErrorInvalidValue;
    const int slots = busiest(mask.live, mask.n);
    return attn_fwd_dispatch(qkv, ldq, o, ldo, lse, batch, tokens, slots > 0 ? slots : 1, 0, mask, s);
}

}  // namespace d2ft

namespace d2ft {

template <typename Mask>
static hipError_t attn_bwd_dispatch(const void* qkv, long ldq, const void* o, long ldo, const float* lse, const void* d_o,
                                    long ld_do, void* dqkv, long ld_dqkv, int batch, int tokens, int n_full,
                                    const Mask& mask, hipStream_t s) {
    if (n_full <= 0) return hipSuccess;
    const bf16* q = static_cast<const bf16*>(qkv);
    const bf16* op = static_cast<const bf16*>(o);
    const bf16* dop = static_cast<const bf16*>(d_o);
    bf16* dq = static_cast<bf16*>(dqkv);
#define D2FT_BWD_CASE(KT) \
    case KT: return launch_bwd_kt<KT, Mask>(q, ldq, op, ldo, lse, dop, ld_do, dq, ld_dqkv, batch, tokens, n_full, mask, s);
    switch ((tokens + 31) / 32) {
        D2FT_BWD_CASE(1) D2FT_BWD_CASE(2) D2FT_BWD_CASE(3) D2FT_BWD_CASE(4)
        D2FT_BWD_CASE(5) D2FT_BWD_CASE(6) D2FT_BWD_CASE(7) D2FT_BWD_CASE(8)
        default: return hipErrorNotSupported;
    }
#undef D2FT_BWD_CASE
}

hipError_t launch_attn_bwd_mfma(const void* qkv, long ldq, const void* o, long ldo, const float* lse, const void* d_o,
                                long ld_do, void* dqkv, long ld_dqkv, int batch, int tokens, int n_full,
                                hipStream_t s) {
    return attn_bwd_dispatch(qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv, ld_dqkv, batch, tokens, n_full, WholeBatch{}, s);
}

hipError_t launch_attn_bwd_mfma_masked(const void* qkv, long ldq, const void* o, long ldo, const float* lse,
                                       const void* d_o, long ld_do, void* dqkv, long ld_dqkv, int batch, int tokens,
                                       int n_full, const MicroMask& mask, hipStream_t s) {
    if (n_full != mask.n_full_pos) return hipErrorInvalidValue;
    if (n_full <= 0) return hipSuccess;
    const int slots = busiest(mask.full, mask.n);
    return attn_bwd_dispatch(qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv, ld_dqkv, batch, tokens, slots > 0 ? slots : 1, mask, s);
}

}  // namespace d2ft
