// Fused softmax attention on the CDNA4 matrix cores for head dimension 64 and up to 256 tokens (forward) or 224 tokens (backward)
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
#include <hip/hip_ext.h>
#include <type_traits>
#include <utility>

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
template <int TP, int NTHR = 256>   // NTHR threads take part, numbered by t (threadIdx.x, or the lane for one wavefront)
__device__ __forceinline__ void load_tile64(const bf16* __restrict__ g, long ld, int rows_valid, bf16* lds, int stride,
                                            int t = threadIdx.x) {
    constexpr int N = TP * 8 / NTHR;
    static_assert(TP * 8 % NTHR == 0, "the tile divides over the threads");
    u32x4 v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = t + i * NTHR;
        const int r = c >> 3, ch = (c & 7) * 8;
        v[i] = u32x4{0u, 0u, 0u, 0u};
        if (r < rows_valid) v[i] = *reinterpret_cast<const u32x4*>(g + (long)r * ld + ch);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = t + i * NTHR;
        *reinterpret_cast<u32x4*>(lds + (c >> 3) * stride + (c & 7) * 8) = v[i];
    }
}
// the same for two tiles at once (K and V): twice the loads in flight
template <int TP, int NTHR = 256>   // NTHR threads take part, numbered by t (threadIdx.x, or the lane for one wavefront)
__device__ __forceinline__ void load_two_tiles64(const bf16* __restrict__ g0, const bf16* __restrict__ g1, long ld,
                                                 int rows_valid, bf16* lds0, int stride0, bf16* lds1, int stride1,
                                                 int t = threadIdx.x) {
    constexpr int N = (TP * 8 + NTHR - 1) / NTHR;
    u32x4 v0[N], v1[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = t + i * NTHR;
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
        const int c = t + i * NTHR;
        if (TP * 8 % NTHR == 0 || c < TP * 8) {
            *reinterpret_cast<u32x4*>(lds0 + (c >> 3) * stride0 + (c & 7) * 8) = v0[i];
            *reinterpret_cast<u32x4*>(lds1 + (c >> 3) * stride1 + (c & 7) * 8) = v1[i];
        }
    }
}

// the same by ONE wavefront with every load of both tiles in flight: raw buffer loads whose declared size
// ends with the last valid row (rows above read as zeros without touching memory), one offset register
// for all chunks (a lane's chunks are 8 rows apart: the distance goes into the scalar offset)
template <int TP>
__device__ __forceinline__ void load_two_tiles64_wave(const bf16* __restrict__ g0, const bf16* __restrict__ g1, long ld,
                                                      int rows_valid, bf16* lds0, int stride0, bf16* lds1, int stride1,
                                                      int lane) {
    constexpr int N = TP * 8 / 64;
    const uint32_t bytes = (uint32_t)(rows_valid - 1) * (uint32_t)ld * 2u + 128u;
    const __amdgpu_buffer_rsrc_t r0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(g0), 0, bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t r1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(g1), 0, bytes, 0x00020000);
    const uint32_t off = (uint32_t)(lane >> 3) * (uint32_t)ld * 2u + (uint32_t)(lane & 7) * 16u;
    const uint32_t step = 8u * (uint32_t)ld * 2u;
    u32x4 v0[N], v1[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        v0[i] = __builtin_amdgcn_raw_buffer_load_b128(r0, off, step * i, 0);
        v1[i] = __builtin_amdgcn_raw_buffer_load_b128(r1, off, step * i, 0);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int c = lane + i * 64;
        *reinterpret_cast<u32x4*>(lds0 + (c >> 3) * stride0 + (c & 7) * 8) = v0[i];
        *reinterpret_cast<u32x4*>(lds1 + (c >> 3) * stride1 + (c & 7) * 8) = v1[i];
    }
}

constexpr int kKS = 72;   // K rows in LDS: 144 bytes (row-form reads)
constexpr int kVS = 96;   // V rows in LDS: 192 bytes (transposing reads)

// ---------------------------------------------------------------------------
// forward: O = softmax(Q K^T / 8) V per (image, live head); log-sum-exp saved for p_f heads
// ---------------------------------------------------------------------------
struct WholeBatch {};   // no mask: every (image, head) pair is live, the first n_full positions are p_f

// One query tile of one pair: S^T = K Q^T against all key tiles, softmax over the keys, O^T = V^T P^T.
// qf: the tile's Q fragments (this lane's query); after_s() runs once the S products are issued (qf is
// free from then on).  Leaves the unnormalised O^T in ot, the row maximum in m, the row sum in sum.
template <int KT, typename AfterS>
__device__ __forceinline__ void fwd_unit(const bf16* Ks, const bf16* Vs, bf16x8 (&qf)[4], int tokens, int lane,
                                         f32x16 (&ot)[2], float& m, float& sum, AfterS&& after_s) {
    const int c = lane & 31, h = lane >> 5;
    // S^T tiles: rows = keys of tile u, column = this lane's query.  K fragments of tile u+1 are
    // fetched from LDS while the MFMAs of tile u run (one read behind each MFMA).
    f32x16 s[KT];
    const f32x16 zero_acc = zero16();   // shared C operand of every tile's first MFMA
    bf16x8 kf[3][4];   // the fragments of a tile are requested two tiles (eight products) before their use
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kf[0][kk] = frag_rows(Ks, kKS, c, kk * 16 + 8 * h);
    if (KT > 1) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kf[1][kk] = frag_rows(Ks, kKS, 32 + c, kk * 16 + 8 * h);
    }
#pragma unroll
    for (int u = 0; u < KT; ++u) {
        if (u + 2 < KT) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kf[(u + 2) % 3][kk] = frag_rows(Ks, kKS, (u + 2) * 32 + c, kk * 16 + 8 * h);
        }
        s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[u % 3][0], qf[0], zero_acc, 0, 0, 0);
#pragma unroll
        for (int kk = 1; kk < 4; ++kk)
            s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[u % 3][kk], qf[kk], s[u], 0, 0, 0);
        if (u + 2 < KT) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    after_s();
    // first V fragments are fetched under the softmax arithmetic
    bf16x8 vf[2][4];
#pragma unroll
    for (int gp = 0; gp < 2; ++gp)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) vf[0][gp * 2 + dt] = frag_tr(Vs, kVS, 16 * gp, dt * 32, lane);
    {   // only the last key tile reaches past the last token (KT = ceil(tokens / 32)): element e of a lane
        // is key 32 (KT - 1) + 8 (e / 4) + 4 h + e % 4
        const int lim = tokens - (KT - 1) * 32 - 4 * h;
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (8 * (e >> 2) + (e & 3) >= lim) s[KT - 1][e] = -INFINITY;
    }
    m = -INFINITY;
#pragma unroll
    for (int u = 0; u < KT; ++u) {
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
    sum = 0.f;
    auto exp_tile = [&](int u) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float p = __builtin_amdgcn_exp2f(fmaf(s[u][e], cexp, -mc));
            s[u][e] = p;
            sum += p;
        }
    };
    exp_tile(0);
    // O^T = V^T P^T: rows = channels, column = this lane's query.  The products of key tile u run on the
    // matrix cores while the vector units take the exponentials of tile u + 1; V fragments one tile ahead.
    ot[0] = zero16();
    ot[1] = zero16();
#pragma unroll
    for (int u = 0; u < KT; ++u) {
        const bf16x8 pf0 = pack8(s[u], 0), pf1 = pack8(s[u], 8);
        if (u + 1 < KT) {
#pragma unroll
            for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
                    vf[(u + 1) & 1][gp * 2 + dt] = frag_tr(Vs, kVS, (u + 1) * 32 + 16 * gp, dt * 32, lane);
        }
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u & 1][dt], pf0, ot[dt], 0, 0, 0);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u & 1][2 + dt], pf1, ot[dt], 0, 0, 0);
        if (u + 1 < KT) {
            exp_tile(u + 1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // one product
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);    // two fragment reads
                __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);   // a quarter of the tile's exponentials
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    sum += __shfl_xor(sum, 32, 64);   // the two lanes of a query hold different keys
}

// A transposed 64 x 32 result (rows = channels in two 32-row halves, column = this lane's token) times mul
// goes to the token's row.  A lane holds 4 consecutive channels per group of 8 and its partner 32 lanes up
// (same token) the other 4: the two exchange halves (v_permlane32_swap), so each stores 16-byte pieces and a
// row goes out as 32 contiguous bytes per store instruction.  All lanes must call; ok says whether this
// lane's token exists.
__device__ __forceinline__ void store_t_rows(const f32x16 (&ot)[2], float mul, bf16* orow, int h, bool ok) {
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            uint32_t a[2], b[2];   // groups 2p and 2p + 1: this lane's 4 channels of each, packed
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                a[r] = pack_bf16x2(ot[dt][8 * p + 2 * r] * mul, ot[dt][8 * p + 2 * r + 1] * mul);
                b[r] = pack_bf16x2(ot[dt][8 * p + 4 + 2 * r] * mul, ot[dt][8 * p + 4 + 2 * r + 1] * mul);
                // upper half of a <-> lower half of b
                const auto sw = __builtin_amdgcn_permlane32_swap(a[r], b[r], false, false);
                a[r] = sw[0];
                b[r] = sw[1];
            }
            // lower lanes now hold channels 8 (2p) .. + 7 (their own 4, then the partner's), upper lanes 8 (2p + 1) .. + 7
            if (ok) *reinterpret_cast<uint4*>(orow + dt * 32 + 8 * (2 * p + h)) = make_uint4(a[0], a[1], b[0], b[1]);
        }
}

// this lane's query row of a forward unit: O = O^T columns / sum, and the log-sum-exp if asked for
__device__ __forceinline__ void fwd_store(const f32x16 (&ot)[2], float m, float sum, bf16* orow, float* lse_q, int h, bool ok) {
    store_t_rows(ot, 1.0f / sum, orow, h, ok);
    if (ok && h == 0 && lse_q) *lse_q = m * kScale + __logf(sum);
}

// the Q fragments of query q (16 bytes per 16-channel step), zeros for a query past the last token
__device__ __forceinline__ void load_q_frags(const bf16* Qb, long ldq, int q, bool q_ok, int h, bf16x8 (&qf)[4]) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (q_ok) v = *reinterpret_cast<const u32x4*>(Qb + (long)q * ldq + kk * 16 + 8 * h);
        qf[kk] = __builtin_bit_cast(bf16x8, v);
    }
}

// which pair a (image, slot) position works on.  Without a mask slot j is live head j and the first n_full
// of them are p_f.  With a mask the position first zero-fills its share of the image's skipped heads (all
// threads of the workgroup), then takes the slot-th live head of the image's micro-batch, if there is one.
template <typename Mask>
__device__ __forceinline__ bool fwd_pair(const Mask& mask, int b, int slot, int n_live, int n_full, int tokens, bf16* o, long ldo,
                                         int& j, bool& save_lse) {
    j = slot;
    save_lse = slot < n_full;
    if constexpr (std::is_same<Mask, MicroMask>::value) {
        const long row0 = (long)b * tokens;
        const int mb = mask.micro_of(b);
        const uint64_t live = mask.live[mb];
        const uint64_t skipped = ~live & (mask.n_live_pos >= 64 ? ~0ull : ((1ull << mask.n_live_pos) - 1ull));
        int r = 0;
        for (uint64_t mm = skipped; mm; mm &= mm - 1, ++r)   // heads skipped in this image's micro-batch: O = 0
            if (r % n_live == slot) {
                const int p = __builtin_ctzll(mm);
                const u32x4 z = {0u, 0u, 0u, 0u};
                for (int i = threadIdx.x; i < tokens * 8; i += blockDim.x)
                    *reinterpret_cast<u32x4*>(o + (row0 + (i >> 3)) * ldo + p * 64 + (i & 7) * 8) = z;
            }
        if (slot >= __builtin_popcountll(live)) return false;
        uint64_t mm = live;
        for (int t = 0; t < slot; ++t) mm &= mm - 1;
        j = __builtin_ctzll(mm);   // this slot's live head
        save_lse = (mask.full[mb] >> j) & 1;
    }
    return true;
}

// One workgroup per (image, slot), four wavefronts that share the query tiles (tokens above 224, where the
// kernel below would need a ninth wavefront).
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
    const long row0 = (long)b * tokens;
    int j;
    bool save_lse;
    if (!fwd_pair(mask, b, blockIdx.x % n_live, n_live, n_full, tokens, o, ldo, j, save_lse)) return;
    const bf16* Qb = qkv + row0 * ldq + j * 192;
    load_two_tiles64<TP>(Qb + 64, Qb + 128, ldq, tokens, Ks, kKS, Vs, kVS);
    __syncthreads();
    for (int qt = wave; qt < KT; qt += 4) {
        const int q = qt * 32 + c;
        const bool q_ok = q < tokens;
        bf16x8 qf[4];
        load_q_frags(Qb, ldq, q, q_ok, h, qf);
        f32x16 ot[2];
        float m, sum;
        fwd_unit<KT>(Ks, Vs, qf, tokens, lane, ot, m, sum, [] {});
        fwd_store(ot, m, sum, o + (row0 + q) * ldo + j * 64, save_lse ? lse + (long)j * rows_total + row0 + q : nullptr, h, q_ok);
    }
}

// Persistent form for up to 224 tokens: a workgroup of KT + 1 wavefronts walks the positions
// blockIdx.x, blockIdx.x + gridDim.x, ... (the grid is what the chip holds at once).  Wavefront t < KT
// owns query tile t of every pair; the last wavefront is the loader: while the others work on pair i out
// of one LDS buffer it copies K and V of pair i + 1 into the other, all its loads in flight at once, so
// after the first pair no wavefront waits for K or V.  A compute wavefront fetches the Q fragments of its
// next pair as soon as the S products of the current one are issued.  One barrier per pair.
template <int KT, typename Mask>
__global__ __launch_bounds__(64 * (KT + 1), 2) void attn_fwd_pipe_kernel(const bf16* __restrict__ qkv, long ldq,
                                                                        bf16* __restrict__ o, long ldo,
                                                                        float* __restrict__ lse, int tokens, int n_live,
                                                                        int n_full, long rows_total, int n_pos,
                                                                        Mask mask) {
    constexpr int TP = KT * 32, NTHR = 64 * (KT + 1);
    constexpr int BUF = TP * (kKS + kVS);   // elements of one K + V buffer
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* const smem = reinterpret_cast<bf16*>(smem_raw);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;

    int pos = blockIdx.x;
    int j = 0;
    bool save_lse = false;
    bool active = fwd_pair(mask, pos / n_live, pos % n_live, n_live, n_full, tokens, o, ldo, j, save_lse);
    {
        const bf16* Qb = qkv + (long)(pos / n_live) * tokens * ldq + j * 192;
        if (active) load_two_tiles64<TP, NTHR>(Qb + 64, Qb + 128, ldq, tokens, smem, kKS, smem + TP * kKS, kVS);
    }
    if (wave == KT) {
        // ---- loader: K and V of the next position into the other buffer, every load in flight at once ----
        __syncthreads();
        for (int i = 0; pos < n_pos; ++i) {
            const int npos = pos + gridDim.x;
            if (npos < n_pos) {
                int nj;
                bool nsave;
                if (fwd_pair(mask, npos / n_live, npos % n_live, n_live, n_full, tokens, o, ldo, nj, nsave)) {
                    const bf16* nQb = qkv + (long)(npos / n_live) * tokens * ldq + nj * 192;
                    bf16* nK = smem + ((i + 1) & 1) * BUF;
                    load_two_tiles64_wave<TP>(nQb + 64, nQb + 128, ldq, tokens, nK, kKS, nK + TP * kKS, kVS, lane);
                }
            }
            __syncthreads();
            pos = npos;
        }
    } else {
        // ---- compute: query tile `wave` of every position ----
        const int q = wave * 32 + c;
        const bool q_ok = q < tokens;
        bf16x8 qf[4];
        if (active) load_q_frags(qkv + (long)(pos / n_live) * tokens * ldq + j * 192, ldq, q, q_ok, h, qf);
        __syncthreads();
        for (int i = 0; pos < n_pos; ++i) {
            const bf16* const Ks = smem + (i & 1) * BUF;
            const bf16* const Vs = Ks + TP * kKS;
            const int npos = pos + gridDim.x;   // the next position of this workgroup (uniform over it)
            int nj = 0;
            bool nsave = false, nactive = false;
            if (npos < n_pos) nactive = fwd_pair(mask, npos / n_live, npos % n_live, n_live, n_full, tokens, o, ldo, nj, nsave);
            const bf16* nQb = qkv + (long)(npos < n_pos ? npos / n_live : 0) * tokens * ldq + nj * 192;
            if (active) {
                const long row0 = (long)(pos / n_live) * tokens;
                f32x16 ot[2];
                float m, sum;
                fwd_unit<KT>(Ks, Vs, qf, tokens, lane, ot, m, sum, [&] {
                    if (nactive) load_q_frags(nQb, ldq, q, q_ok, h, qf);
                });
                fwd_store(ot, m, sum, o + (row0 + q) * ldo + j * 64, save_lse ? lse + (long)j * rows_total + row0 + q : nullptr, h, q_ok);
            } else if (nactive) {
                load_q_frags(nQb, ldq, q, q_ok, h, qf);
            }
            __syncthreads();
            pos = npos;
            j = nj;
            save_lse = nsave;
            active = nactive;
        }
    }
}

template <int KT, typename Mask>
hipError_t launch_fwd_kt(const bf16* qkv, long ldq, bf16* o, long ldo, float* lse, int batch, int tokens, int n_live,
                         int n_full, const Mask& mask, hipStream_t s) {
    if constexpr (KT <= 7) {
        constexpr size_t lds = 2 * (size_t)KT * 32 * (kKS + kVS) * sizeof(bf16);
        constexpr int threads = 64 * (KT + 1);
        auto kern = attn_fwd_pipe_kernel<KT, Mask>;
        static int resident = 0;   // workgroups the chip holds at once
        if (resident == 0) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            int dev = 0, cus = 0, per_cu = 0;
            if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
            if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
            if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, threads, lds)) != hipSuccess) return e;
            resident = cus * (per_cu < 1 ? 1 : per_cu);
        }
        const int n_pos = batch * n_live;
        // every workgroup gets the same number of positions, give or take one
        const int rounds = (n_pos + resident - 1) / resident;
        const int grid = (n_pos + rounds - 1) / rounds;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds, s, qkv, ldq, o, ldo, lse, tokens, n_live, n_full,
                           (long)batch * tokens, n_pos, mask);
        return hipGetLastError();
    } else {
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
}

// ---------------------------------------------------------------------------
// backward for p_f heads: dQ, dK, dV from Q, K, V, O, dO and the saved log-sum-exp
//
// Per 32x32 tile pair (query tile i, key tile u), in the orientation S = Q K^T (a lane owns one KEY
// column, its 16 result elements are 16 queries):
//     S  = Q_i K_u^T              P  = exp(S/8 - lse_q)          (probabilities are rebuilt, never stored)
//     dP = dO_i V_u^T             dS = P * (dP - delta_q),       delta_q = sum_d dO[q][d] O[q][d]
//     dV_u^T += dO_i^T P          dK_u^T += Q_i^T dS             (P, dS feed the MFMA straight from registers)
//     dQ_i^T  = sum_u K_u^T dS_iu^T
// The workgroup has KT + 1 wavefronts.  Wavefront u < KT owns key tile u: it holds the K_u and V_u
// operand fragments and its dK, dV accumulators in registers for the whole kernel, walks the query
// tiles and leaves each dS_iu (bf16, 2 KB) in LDS.  Its loop is software-pipelined: the S and dP
// products of query tile i + 1 are issued before the exponentials of tile i, so the matrix cores work
// under the vector arithmetic.  The last wavefront owns dQ: one step behind the others it multiplies
// the KT tiles dS_iu of a query tile with K^T out of LDS, so dQ_i is MFMA chains in a fixed order - no
// partial sums cross wavefronts - and goes from its registers to memory.  Query tiles (Q_i, dO_i) are
// triple-buffered and the dS tiles double-buffered in LDS, which leaves one barrier per query tile.
// The per-query constants ride in the products: a query row of Q carries -8 lse_q and a row of dO
// carries -delta_q (each split into two bf16 terms) in two extra channels that meet a 1 on the K / V
// side, so the MFMAs deliver S - 8 lse and dP - delta and the lanes read no per-query values from LDS.
// If bsum is given the kernel also writes the column sums of the pair's dQ, dK, dV rows (the
// gradient of the QKV bias: one row of 192 partial sums per image).
// ---------------------------------------------------------------------------
constexpr int kTS = 104;   // K rows, read both ways once (row-form and transposing): 208 bytes
// Query tiles (Q_i, dO_i) are read both ways in every step.  A 128-bit row-form read is free of bank conflicts
// when eight consecutive rows start in different 16-byte slots of a 128-byte line (row stride an odd multiple
// of 16 bytes); a transposing read when the four rows of a 16-lane group start 32 bytes apart modulo 128.  No
// stride does both for rows in their natural order, so row r of every group of eight is kept at position
// (0, 2, 4, 6, 1, 3, 5, 7)[r % 8] with a stride of 176 bytes: eight rows still start in eight different slots,
// and rows r .. r + 3 of a half group sit two strides apart, i.e. 96 bytes modulo 128.
constexpr int kQS = 88;
__device__ __forceinline__ int tile_row(int r) { return (r & ~7) | ((r & 3) << 1) | ((r >> 2) & 1); }
// the transposing read of frag_tr for such a tile: logical rows t0 + 4h + {0..3} and t0 + 8 + 4h + {0..3}
__device__ __forceinline__ bf16x8 frag_tr_tile(const bf16* lds, int t0, int ch0, int lane) {
    const int j = lane & 15;
    const bf16* p = lds + (t0 + 2 * (j >> 2) + (lane >> 5)) * kQS + ch0 + 16 * ((lane >> 4) & 1) + 4 * (j & 3);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 8 * kQS));
    s16x8 r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return __builtin_bit_cast(bf16x8, r);
}
// dS tiles [32 keys][32 queries]: rows of 96 bytes, so that the four key rows of a transposing read start
// 32 bytes apart modulo 128
constexpr int kDS = 48;

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop whose index is a compile-time constant
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int KT, typename Mask>
__global__ __launch_bounds__(64 * (KT + 1)) void attn_bwd_mfma_kernel(const bf16* __restrict__ qkv, long ldq,
                                                                      const bf16* __restrict__ o, long ldo,
                                                                      const float* __restrict__ lse,
                                                                      const bf16* __restrict__ d_o, long ld_do,
                                                                      bf16* __restrict__ dqkv, long ld_dqkv,
                                                                      float* __restrict__ bsum, long ld_bsum,
                                                                      int tokens, int n_full, long rows_total,
                                                                      Mask mask) {
    constexpr int TP = KT * 32;
    constexpr int NTHR = 64 * (KT + 1);
    constexpr int NLD = (512 + NTHR - 1) / NTHR;         // 16-byte chunks of a (Q_i, dO_i) tile pair per thread
    constexpr int NDL = (TP * 8 + NTHR - 1) / NTHR;      // (query, 16-byte piece) items of the delta sums per thread
    constexpr int NKL = (TP * 8 + NTHR - 1) / NTHR;      // 16-byte chunks of K per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* Ks = reinterpret_cast<bf16*>(smem_raw);        // [TP][kTS]      read transposed by the dQ wavefront
    bf16* Qs = Ks + TP * kTS;                            // [3][32][kQS]   query tile i in buffer i % 3, rows permuted
    bf16* dOs = Qs + 3 * 32 * kQS;                       // [3][32][kQS]
    bf16* dSs_all = dOs + 3 * 32 * kQS;                  // [2][KT][32 keys][kDS]
    float* lse_s = reinterpret_cast<float*>(dSs_all + 2 * KT * 32 * kDS);   // [TP]   -8 lse_q
    float* del_s = lse_s + TP;                           // [TP]   -delta_q
    bf16* dq_stage = reinterpret_cast<bf16*>(del_s + TP);   // [32][72]   the dQ wavefront's store staging
    float* red = reinterpret_cast<float*>(dq_stage + 32 * 72);   // [KT][128]   column sums of dK, dV per key tile
    float* sk_s = red + KT * 128;                        // [TP]   sum over the queries of dS[q][key], for dQ's column sums
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
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
                const int p = __builtin_ctzll(m);
                bf16* zb = dqkv + row0 * ld_dqkv + p * 192;
                const u32x4 z = {0u, 0u, 0u, 0u};
                for (int i = threadIdx.x; i < tokens * 24; i += NTHR)
                    *reinterpret_cast<u32x4*>(zb + (long)(i / 24) * ld_dqkv + (i % 24) * 8) = z;
                if (bsum)
                    for (int i = threadIdx.x; i < 192; i += NTHR) bsum[(long)b * ld_bsum + p * 192 + i] = 0.f;
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
    const int u = wave;                 // this wavefront's key tile (wave == KT: the dQ wavefront)
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    // ---- prologue: every global load of it is issued before the first use of any ----
    // chunk id = threadIdx.x + k * NTHR of the 512 chunks of (Q_i, dO_i): ids below 256 are Q's
    auto fetch_tile = [&](int i, u32x4 (&nx)[NLD]) {
#pragma unroll
        for (int k = 0; k < NLD; ++k) {
            const int id = threadIdx.x + k * NTHR;
            const int t = id & 255, r = t >> 3, ch = (t & 7) * 8;
            const int q = i * 32 + r;
            nx[k] = zero4;
            if (id < 512 && i < KT && q < tokens)
                nx[k] = (id < 256) ? *reinterpret_cast<const u32x4*>(Qb + (long)q * ldq + ch)
                                   : *reinterpret_cast<const u32x4*>(dOb + (long)q * ld_do + ch);
        }
    };
    // channels 64 .. 79 of a tile row: the row's constant as two bf16 terms (a = hi + lo), then zeros
    auto store_extra = [&](bf16* row, float a) {
        const __bf16 hi = static_cast<__bf16>(a);
        const __bf16 lo = static_cast<__bf16>(a - static_cast<float>(hi));
        typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
        bf16x2_t t2;
        t2[0] = hi;
        t2[1] = lo;
        const u32x4 first = {__builtin_bit_cast(uint32_t, t2), 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(row + 64) = first;
        *reinterpret_cast<u32x4*>(row + 72) = zero4;
    };
    auto store_tile = [&](int i, const u32x4 (&nx)[NLD], bool extra) {   // into buffer i % 3
#pragma unroll
        for (int k = 0; k < NLD; ++k) {
            const int id = threadIdx.x + k * NTHR;
            const int t = id & 255;
            bf16* dst = (id < 256 ? Qs : dOs) + (i % 3) * 32 * kQS + tile_row(t >> 3) * kQS + (t & 7) * 8;
            if (id < 512) *reinterpret_cast<u32x4*>(dst) = nx[k];
        }
        if (extra && threadIdx.x < 64) {   // the constants of tile i's 32 queries: Q rows, then dO rows
            const int r = threadIdx.x & 31;
            const bool is_q = threadIdx.x < 32;
            store_extra((is_q ? Qs : dOs) + (i % 3) * 32 * kQS + tile_row(r) * kQS, (is_q ? lse_s : del_s)[i * 32 + r]);
        }
    };
    // V operand fragments of this wavefront's key tile: rows u*32 + c of V, 8 channels at kk*16 + 8h
    bf16x8 kfr[5], vfr[5];
    {
        typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
        const short one = h == 0 ? (short)0x3F80 : (short)0;   // bf16 1.0 against the two extra channels
        const s16x8_t ones = {one, one, 0, 0, 0, 0, 0, 0};
        kfr[4] = vfr[4] = __builtin_bit_cast(bf16x8, ones);
    }
    {
        const int key = u * 32 + c;
        const bool ok = wave < KT && key < tokens;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4 v = zero4;
            if (ok) v = *reinterpret_cast<const u32x4*>(Qb + 128 + (long)key * ldq + kk * 16 + 8 * h);
            vfr[kk] = __builtin_bit_cast(bf16x8, v);
        }
    }
    // query tiles in flight from memory: tile t sits in ring slot t % kAhead from its fetch until it is stored to
    // LDS kAhead steps later (memory latency is several steps long)
    constexpr int kAhead = 3;
    u32x4 kl[NKL], da[NDL], dg[NDL], nx0[NLD], nx1[NLD], ring[kAhead][NLD];
#pragma unroll
    for (int k = 0; k < NKL; ++k) {
        const int id = threadIdx.x + k * NTHR;
        const int r = id >> 3, ch = (id & 7) * 8;
        kl[k] = zero4;
        if (r < tokens) kl[k] = *reinterpret_cast<const u32x4*>(Qb + 64 + (long)r * ldq + ch);   // r < tokens <= TP
    }
    fetch_tile(0, nx0);
    fetch_tile(1, nx1);
#pragma unroll
    for (int t = 2; t < 2 + kAhead; ++t) fetch_tile(t, ring[t % kAhead]);
#pragma unroll
    for (int k = 0; k < NDL; ++k) {
        const int it = threadIdx.x + k * NTHR;
        const int q = it >> 3, ch = (it & 7) * 8;
        da[k] = dg[k] = zero4;
        if (q < tokens) {
            da[k] = *reinterpret_cast<const u32x4*>(dOb + (long)q * ld_do + ch);
            dg[k] = *reinterpret_cast<const u32x4*>(Ob + (long)q * ldo + ch);
        }
    }
    float lq[(TP + NTHR - 1) / NTHR];
#pragma unroll
    for (int k = 0; k < (TP + NTHR - 1) / NTHR; ++k) {
        const int q = threadIdx.x + k * NTHR;
        lq[k] = q < tokens ? lse[(long)j * rows_total + row0 + q] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < NKL; ++k) {
        const int id = threadIdx.x + k * NTHR;
        if (id < TP * 8) *reinterpret_cast<u32x4*>(Ks + (id >> 3) * kTS + (id & 7) * 8) = kl[k];
    }
    store_tile(0, nx0, false);
    store_tile(1, nx1, false);
    // delta_q = sum_d dO[q][d] O[q][d]: eight lanes per query, one 16-byte piece of the row each
#pragma unroll
    for (int k = 0; k < NDL; ++k) {
        const int it = threadIdx.x + k * NTHR;
        float dl = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dl = fmaf(__uint_as_float(da[k][i] << 16), __uint_as_float(dg[k][i] << 16), dl);
            dl = fmaf(__uint_as_float(da[k][i] & 0xffff0000u), __uint_as_float(dg[k][i] & 0xffff0000u), dl);
        }
        dl += __shfl_xor(dl, 1, 64);
        dl += __shfl_xor(dl, 2, 64);
        dl += __shfl_xor(dl, 4, 64);
        if ((it & 7) == 0 && it < TP * 8) {
            const int q = it >> 3;
            del_s[q] = -dl;
            if (q < 64) store_extra(dOs + (q >> 5) * 32 * kQS + tile_row(q & 31) * kQS, -dl);   // tiles 0 and 1 are in LDS already
        }
    }
#pragma unroll
    for (int k = 0; k < (TP + NTHR - 1) / NTHR; ++k) {
        const int q = threadIdx.x + k * NTHR;
        if (q < TP) {
            sk_s[q] = 0.f;
            lse_s[q] = -8.f * lq[k];
            if (q < 64) store_extra(Qs + (q >> 5) * 32 * kQS + tile_row(q & 31) * kQS, -8.f * lq[k]);
        }
    }
    __syncthreads();
    const float cexp = kScale * kLog2e;
    // LDS area in which a wavefront turns a transposed [64 channels][32 rows] result into 16-byte row pieces
    // ([32][72] bf16): the dQ wavefront has its own; the key wavefronts use theirs once, after the last step,
    // in the space of the query tiles
    bf16* const stage = wave < KT ? Qs + wave * (32 * 72) : dq_stage;
    float* const bout = bsum ? bsum + (long)b * ld_bsum + j * 192 : nullptr;

    // The two kinds of wavefront run their own copy of the step loop (each keeps a different set of values in
    // registers for the whole kernel); both copies meet the same barriers.
    if (wave < KT) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kfr[kk] = frag_rows(Ks, kTS, u * 32 + c, kk * 16 + 8 * h);
        f32x16 dKt[2], dVt[2];   // dK^T and dV^T of the key tile: rows = channels, column = key c
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
            dKt[dt] = zero16();
            dVt[dt] = zero16();
        }
        const float key_on = (u * 32 + c) < tokens ? 1.f : 0.f;   // keys beyond the last token: P = 0
        // S - 8 lse of query tile t against this wavefront's key tile (kept for two steps: [t & 1])
        f32x16 sc[2];
        {
            f32x16 s0 = zero16();
#pragma unroll
            for (int kk = 0; kk < 5; ++kk)
                s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Qs, kQS, tile_row(c), kk * 16 + 8 * h), kfr[kk], s0, 0, 0, 0);
            sc[0] = s0;
        }
        static_for<KT + 1>([&](auto step_index) {
            constexpr int i = decltype(step_index)::value;
            if (i > 0) __syncthreads();   // every wavefront is done with step i - 1
            if (i + 2 < KT) {   // tile i + 2 is read from the next step on; its buffer held tile i - 1
                store_tile(i + 2, ring[(i + 2) % kAhead], true);
                fetch_tile(i + 2 + kAhead, ring[(i + 2) % kAhead]);
            }
            if (i < KT) {
                // Issue order of a step: all fragment reads; dP of this tile and S of the next one on the matrix
                // cores with the exponentials of this tile's S (computed one step ago) between them on the vector
                // ALUs; dV with dS and its hand-over between the MFMAs; dK, which runs under the next step's reads.
                const bf16* Qi = Qs + (i % 3) * 32 * kQS;
                const bf16* dOi = dOs + (i % 3) * 32 * kQS;
                const bf16* Qn = Qs + ((i + 1) % 3) * 32 * kQS;
                bf16x8 dof[5], qnf[5], dot[2][2], qt[2][2];
#pragma unroll
                for (int kk = 0; kk < 5; ++kk) dof[kk] = frag_rows(dOi, kQS, tile_row(c), kk * 16 + 8 * h);
                if (i + 1 < KT) {
#pragma unroll
                    for (int kk = 0; kk < 5; ++kk) qnf[kk] = frag_rows(Qn, kQS, tile_row(c), kk * 16 + 8 * h);
                }
#pragma unroll
                for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        dot[gp][dt] = frag_tr_tile(dOi, 16 * gp, dt * 32, lane);
                        qt[gp][dt] = frag_tr_tile(Qi, 16 * gp, dt * 32, lane);
                    }
                __builtin_amdgcn_sched_barrier(0);
                f32x16 dp = zero16(), sn = zero16();   // dP - delta, and S - 8 lse of the next tile
                f32x16& s = sc[i & 1];
#pragma unroll
                for (int kk = 0; kk < 5; ++kk) {
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dof[kk], vfr[kk], dp, 0, 0, 0);
                    if (i + 1 < KT) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qnf[kk], kfr[kk], sn, 0, 0, 0);
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) s[e] = __builtin_amdgcn_exp2f(s[e] * cexp) * key_on;   // P
                bf16x8 pf[2];
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) pf[gp] = pack8(s, 8 * gp);
                {
                    constexpr int NM = 5 + (i + 1 < KT ? 5 : 0);   // MFMAs of this phase; 56 vector ALU instructions
#pragma unroll
                    for (int k = 0; k < NM; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, (56 + NM - 1) / NM, 0);
                    }
                }
                if (i + 1 < KT) sc[(i + 1) & 1] = sn;
                __builtin_amdgcn_sched_barrier(0);
                bf16* dSs = dSs_all + ((i & 1) * KT + wave) * 32 * kDS;
                f32x16 ds;
                bf16x8 dsf[2];
#pragma unroll
                for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
                        dVt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot[gp][dt], pf[gp], dVt[dt], 0, 0, 0);
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    // element e = 4 * eg + k is query 8 * eg + 4 * h + k of the tile
#pragma unroll
                    for (int k = 0; k < 4; ++k) ds[4 * eg + k] = s[4 * eg + k] * dp[4 * eg + k];
                    // hand dS to the dQ wavefront: [key][query] tile, 8-byte writes
                    uint2 pk;
                    pk.x = pack_bf16x2(ds[4 * eg], ds[4 * eg + 1]);
                    pk.y = pack_bf16x2(ds[4 * eg + 2], ds[4 * eg + 3]);
                    *reinterpret_cast<uint2*>(dSs + c * kDS + 8 * eg + 4 * h) = pk;
                }
#pragma unroll
                for (int gp = 0; gp < 2; ++gp) dsf[gp] = pack8(ds, 8 * gp);
#pragma unroll
                for (int k = 0; k < 4; ++k) {   // 4 MFMAs; 16 products, 16 conversions, 4 stores
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
                        dKt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt[gp][dt], dsf[gp], dKt[dt], 0, 0, 0);
                if (bsum) {   // uniform over the grid
                    // the dS values as the dQ wavefront multiplies them (bf16), added over this lane's 16 queries
                    // under the products above and then to the key's running sum in LDS (both lanes of a key add)
                    float t = 0.f;
#pragma unroll
                    for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                        for (int k = 0; k < 8; ++k) t += static_cast<float>(dsf[gp][k]);
                    atomicAdd(sk_s + u * 32 + c, t);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        // The column sums of dQ = (1/8) dS K follow from the query sums of dS: sum_q dQ[q][d] = (1/8) sum_k sk[k] K[k][d];
        // the dQ wavefront forms them from the sums in sk_s while the key wavefronts store dK and dV.
        __syncthreads();   // the query tiles are free
        // dK^T: straight from the accumulators, 16-byte pieces after a half-wave exchange.  Its column sums are
        // not formed: sum_k dK[k][.] = (1/8) sum_q (sum_k dS[q][k]) Q[q][.] and sum_k dS[q][k] = sum_k P dP - delta_q = 0
        // (softmax does not see a shift of all keys), so the key bias gradient is written as the zero it is.
        store_t_rows(dKt, kScale, dQb + (long)(u * 32 + c) * ld_dqkv + 64, h, u * 32 + c < tokens);
        if (!bsum) {
            store_t_rows(dVt, 1.f, dQb + (long)(u * 32 + c) * ld_dqkv + 128, h, u * 32 + c < tokens);
        } else {
            // dV^T through the wavefront's LDS area, where its column sums are taken
            constexpr int m = 1;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    uint2 pk;
                    pk.x = pack_bf16x2(dVt[dt][4 * eg], dVt[dt][4 * eg + 1]);
                    pk.y = pack_bf16x2(dVt[dt][4 * eg + 2], dVt[dt][4 * eg + 3]);
                    *reinterpret_cast<uint2*>(stage + c * 72 + dt * 32 + 8 * eg + 4 * h) = pk;
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int id = lane + 64 * k, r = id >> 3, ch = (id & 7) * 8;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stage + r * 72 + ch);
                const int key = u * 32 + r;
                if (key < tokens) *reinterpret_cast<u32x4*>(dQb + (long)key * ld_dqkv + 64 + 64 * m + ch) = v;
            }
            {
                // Column sums of the staged tile (the values as they are stored; rows beyond the last token are
                // zero): lane (p = lane % 32, half = lane / 32) adds channels 2p, 2p + 1 over rows 16 half .. + 15
                float s0 = 0.f, s1 = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t w = *reinterpret_cast<const uint32_t*>(stage + (16 * h + r) * 72 + 2 * c);
                    s0 += __uint_as_float(w << 16);
                    s1 += __uint_as_float(w & 0xffff0000u);
                }
                s0 += __shfl_xor(s0, 32, 64);
                s1 += __shfl_xor(s1, 32, 64);
                if (h == 0) {
                    red[wave * 128 + 64 * m + 2 * c] = s0;
                    red[wave * 128 + 64 * m + 2 * c + 1] = s1;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (bsum) __syncthreads();   // the per-tile sums are complete
    } else {
        // the dQ wavefront keeps all of K^T as operand fragments: [key tile][16-key half][channel half]
        bf16x8 ktf[KT][2][2];
#pragma unroll
        for (int v = 0; v < KT; ++v)
#pragma unroll
            for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) ktf[v][gp][dt] = frag_tr(Ks, kTS, v * 32 + 16 * gp, dt * 32, lane);
#pragma unroll
        for (int i = 0; i <= KT; ++i) {
            if (i > 0) __syncthreads();   // the dS tiles of query tile i - 1 are visible
            if (i + 2 < KT) {
                store_tile(i + 2, ring[(i + 2) % kAhead], true);
                fetch_tile(i + 2 + kAhead, ring[(i + 2) % kAhead]);
            }
            if (i >= 1) {
                // dQ^T of query tile i - 1: rows = channels, column = query c; four MFMA chains (channel half x
                // 16-key half), added pairwise at the end.  All dS fragments of the query tile are requested from
                // LDS before the first product: this wavefront's step is the longest of the workgroup.
                const int t = i - 1;
                const bf16* dSt = dSs_all + ((t & 1) * KT) * 32 * kDS;
                f32x16 acc[2][2] = {{zero16(), zero16()}, {zero16(), zero16()}};
                bf16x8 dsf[KT][2];   // [key tile][16-key half]
#pragma unroll
                for (int v = 0; v < KT; ++v)
#pragma unroll
                    for (int gp = 0; gp < 2; ++gp)
                        dsf[v][gp] = frag_tr(dSt + v * 32 * kDS, kDS, 16 * gp, 0, lane);   // column = query c, slots = keys
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int v = 0; v < KT; ++v) {
#pragma unroll
                    for (int gp = 0; gp < 2; ++gp)
#pragma unroll
                        for (int dt = 0; dt < 2; ++dt)
                            acc[gp][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf[v][gp][dt], dsf[v][gp], acc[gp][dt], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                // straight from the accumulators: 16-byte pieces after a half-wave exchange
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[0][dt][e] += acc[1][dt][e];
                store_t_rows(acc[0], kScale, dQb + (long)(t * 32 + c) * ld_dqkv, h, t * 32 + c < tokens);
            }
        }
        __syncthreads();   // matches the key wavefronts' barrier before their stores; their sk are visible
        if (bsum) {
            // sum_k sk[k] K[k][.]: lane (piece = lane % 8, part = lane / 8) takes channels 8 piece .. + 7 of the keys
            // k = part, part + 8, ...; the eight parts are added in lane order
            float a8[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) a8[i] = 0.f;
            const int piece = lane & 7, part = lane >> 3;
#pragma unroll 4
            for (int k = part; k < TP; k += 8) {   // rows of K beyond the last token are zero
                const u32x4 kv = *reinterpret_cast<const u32x4*>(Ks + k * kTS + piece * 8);
                const float w = sk_s[k];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a8[2 * i] = fmaf(w, __uint_as_float(kv[i] << 16), a8[2 * i]);
                    a8[2 * i + 1] = fmaf(w, __uint_as_float(kv[i] & 0xffff0000u), a8[2 * i + 1]);
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float t = a8[i];
                t += __shfl_xor(t, 8, 64);
                t += __shfl_xor(t, 16, 64);
                t += __shfl_xor(t, 32, 64);
                a8[i] = t * kScale;
            }
            if (part == 0) store8(bout + piece * 8, a8);
            __syncthreads();
        }
    }
    if (bsum && threadIdx.x < 128) {   // dK sums (zero) and dV sums: key tiles added in index order
        float t = 0.f;
        if (threadIdx.x >= 64) {
#pragma unroll
            for (int v = 0; v < KT; ++v) t += red[v * 128 + threadIdx.x];
        }
        bout[64 + threadIdx.x] = t;
    }
}

template <int KT>
constexpr size_t bwd_lds_bytes() {
    constexpr int TP = KT * 32;
    static_assert(KT * 32 * 72 <= 6 * 32 * kQS, "the key wavefronts' store staging fits the query tiles' space");
    constexpr size_t tiles = (size_t)(TP * kTS + 6 * 32 * kQS + 2 * KT * 32 * kDS + 32 * 72) * sizeof(bf16) +
                             (size_t)(3 * TP + KT * 128) * sizeof(float);
    return tiles;
}

template <int KT, typename Mask>
hipError_t launch_bwd_kt(const bf16* qkv, long ldq, const bf16* o, long ldo, const float* lse, const bf16* d_o, long ld_do,
                         bf16* dqkv, long ld_dqkv, float* bsum, long ld_bsum, int batch, int tokens, int n_full,
                         const Mask& mask, hipStream_t s) {
    constexpr size_t lds = bwd_lds_bytes<KT>();
    static_assert(lds <= 160 * 1024, "the pair's tiles must fit a compute unit's LDS");
    auto kern = attn_bwd_mfma_kernel<KT, Mask>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (hipEvent_t ev = launch_signal_take()) {   // the launch completes the event itself
        hipExtLaunchKernelGGL(kern, dim3(batch * n_full), dim3(64 * (KT + 1)), lds, s, nullptr, ev, 0, qkv, ldq, o, ldo, lse,
                              d_o, ld_do, dqkv, ld_dqkv, bsum, ld_bsum, tokens, n_full, (long)batch * tokens, mask);
    } else {
        hipLaunchKernelGGL(kern, dim3(batch * n_full), dim3(64 * (KT + 1)), lds, s, qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv,
                           ld_dqkv, bsum, ld_bsum, tokens, n_full, (long)batch * tokens, mask);
    }
    return hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(int tokens, long ldq, long ldo) {
    return tokens >= 1 && tokens <= 256 && (ldq % 8) == 0 && (ldo % 8) == 0;
}
// The backward keeps one wavefront per 32-key tile plus one for dQ at up to 256 registers each, which a
// compute unit holds for at most seven key tiles.
bool attn_bwd_mfma_supported(int tokens, long ldq, long ldo) {
    return attn_mfma_supported(tokens, ldq, ldo) && tokens <= 224;
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
                                    long ld_do, void* dqkv, long ld_dqkv, float* bsum, long ld_bsum, int batch, int tokens,
                                    int n_full, const Mask& mask, hipStream_t s) {
    if (n_full <= 0) return hipSuccess;
    const bf16* q = static_cast<const bf16*>(qkv);
    const bf16* op = static_cast<const bf16*>(o);
    const bf16* dop = static_cast<const bf16*>(d_o);
    bf16* dq = static_cast<bf16*>(dqkv);
#define D2FT_BWD_CASE(KT) \
    case KT: return launch_bwd_kt<KT, Mask>(q, ldq, op, ldo, lse, dop, ld_do, dq, ld_dqkv, bsum, ld_bsum, batch, tokens, n_full, mask, s);
    switch ((tokens + 31) / 32) {
        D2FT_BWD_CASE(1) D2FT_BWD_CASE(2) D2FT_BWD_CASE(3) D2FT_BWD_CASE(4)
        D2FT_BWD_CASE(5) D2FT_BWD_CASE(6) D2FT_BWD_CASE(7)
        default: return hipErrorNotSupported;
    }
#undef D2FT_BWD_CASE
}

hipError_t launch_attn_bwd_mfma(const void* qkv, long ldq, const void* o, long ldo, const float* lse, const void* d_o,
                                long ld_do, void* dqkv, long ld_dqkv, float* bsum, long ld_bsum, int batch, int tokens,
                                int n_full, hipStream_t s) {
    return attn_bwd_dispatch(qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv, ld_dqkv, bsum, ld_bsum, batch, tokens, n_full,
                             WholeBatch{}, s);
}

hipError_t launch_attn_bwd_mfma_masked(const void* qkv, long ldq, const void* o, long ldo, const float* lse,
                                       const void* d_o, long ld_do, void* dqkv, long ld_dqkv, float* bsum, long ld_bsum,
                                       int batch, int tokens, int n_full, const MicroMask& mask, hipStream_t s) {
    if (n_full != mask.n_full_pos) return hipErrorInvalidValue;
    if (n_full <= 0) return hipSuccess;
    const int slots = busiest(mask.full, mask.n);
    return attn_bwd_dispatch(qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv, ld_dqkv, bsum, ld_bsum, batch, tokens,
                             slots > 0 ? slots : 1, mask, s);
}

}  // namespace d2ft
