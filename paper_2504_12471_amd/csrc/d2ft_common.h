// Internal declarations shared by the HIP sources of libd2ft (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/d2ft.h"

namespace d2ft {

typedef __bf16 bf16;

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kHeadDim = 64;
constexpr int kMaxBlocks64 = 3 * D2FT_MAX_HEADS;   // 64-row blocks of a compacted QKV weight

// ---------------------------------------------------------------------------
// element access: storage type T (float or bf16), arithmetic in float
// ---------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ float ld(const T* p) { return static_cast<float>(*p); }
template <typename T> __device__ __forceinline__ void st(T* p, float v) { *p = static_cast<T>(v); }

// 8 consecutive elements; p must be aligned to 8 elements
__device__ __forceinline__ void load8(const float* p, float (&o)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16* p, float (&o)[8]) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[2 * i] = __uint_as_float(w[i] << 16);
        o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    bf16x2_t t;
    t[0] = static_cast<__bf16>(lo);
    t[1] = static_cast<__bf16>(hi);
    return __builtin_bit_cast(uint32_t, t);
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
    uint4 r;
    r.x = pack_bf16x2(v[0], v[1]);
    r.y = pack_bf16x2(v[2], v[3]);
    r.z = pack_bf16x2(v[4], v[5]);
    r.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = r;
}

// ---------------------------------------------------------------------------
// wavefront reductions (all 64 lanes take part and receive the result)
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// exact (erf) GELU and its derivative
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_f(float z) {
    const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
    const float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
    return cdf + z * pdf;
}

// ---------------------------------------------------------------------------
// 64-granular index remap: a compacted index i maps to tbl[i / 64] + i % 64.
// It turns "column c of the compacted live-head layout" into a row or column
// of the full weight tensor.
// ---------------------------------------------------------------------------
struct Remap64 {
    int32_t start[kMaxBlocks64];
    __host__ __device__ __forceinline__ int operator()(int i) const { return start[i >> 6] + (i & 63); }
};

// ---------------------------------------------------------------------------
// GEMM problem: C[m][n] = epilogue( sum_k A(m,k) * B(k,n) )
//   A(m,k) = A[m*a_rs + k*a_cs],  B(k,n) = B[k*b_rs + n*b_cs]   (element strides)
// ---------------------------------------------------------------------------
enum { REMAP_NONE = 0, REMAP_B_N = 1, REMAP_B_K = 2 };
// kernel instantiations only: REMAP_B_K whose K walk is cut down per tile row to the 64-wide blocks of the
// positions that take part in a row segment the tile overlaps (launch_gemm_mfma_kseg)
constexpr int REMAP_B_KSEG = 3;
enum { ACT_NONE = 0, ACT_GELU = 1, ACT_DGELU = 2 };

// One problem of a grouped weight-gradient launch: C_g[m][n] = sum_k A_g[k][m] * B_g[k][n], k over the token
// rows (both operands stored with k strided: lda, ldb are the row strides in elements)
struct GemmGroup {
    const void* A;
    const void* B;
    long lda, ldb;
    int M, N;
    int tiles_m, tile0;   // 256-row tiles of this problem; index of its first tile in the launch's tile list
};
constexpr int kMaxGemmGroups = 4;

// Row segments of a GEMM whose output columns come in "positions" of `slice` columns, with a set of positions
// per segment that take part (micro-batches with their own op codes over gated feed-forward slices): an
// output element of a row in segment i and a column of position p is computed if bit p of pos[i] is set and
// written as zero otherwise.  launch_gemm_mfma_seg skips the 256x256 tiles no row of which takes part (they are
// only zero-filled) and deals the tiles with work evenly over the workgroups.
// The same description serves a GEMM whose *K* index comes in positions (launch_gemm_mfma_kseg): the columns of A
// at position p are zero in the rows of a segment in which p does not take part; every segment gets tile rows of
// its own (row_before[i]: the first tile row of segment i, live_tiles: their number) and a tile walks only the
// positions of its segment.
constexpr int kMaxGemmSegments = 8;
constexpr int kMaxSegTileRows = 64;
struct GemmRowSegments {
    int n;                               // 0: not in use
    int slice;                           // columns per position, a multiple of 64
    int end[kMaxGemmSegments];           // row ends, ascending; the last is M
    uint64_t pos[kMaxGemmSegments];
    // filled by the launcher, for 256 x 256 tiles
    int live_tiles;
    uint16_t row_live[kMaxSegTileRows];        // tile row t: bit j = column tile j has work in a segment the row overlaps
    uint16_t row_before[kMaxSegTileRows + 1];  // tiles with work in the tile rows before t
    uint8_t pos_segs[64];                      // position p: bit i = it takes part in segment i
};

struct GemmArgs {
    const void* A;
    const void* B;
    void* C;
    long a_rs, a_cs, b_rs, b_cs, ldc;
    int M, N, K;
    int remap;            // REMAP_*: which index of B goes through tbl
    int bias_remap;       // bias index n goes through tbl
    const void* bias;     // [N] or null
    const void* residual; // [M][ldr] or null, added in the epilogue
    long ldr;
    int act;              // ACT_GELU: Z <- gelu'(z), C <- gelu(z), z = the fp32 pre-activation; ACT_DGELU: C <- acc * Z
    void* Z;
    long ldz;
    float* partial;       // non-null: split-K mode, raw fp32 sums go to partial[split][M][N]
    int splits;
    int tile_hint;        // 0: kernel chooses its tile, 1: 256x256, 2: 128x128, 3: 192x256
    // grouped mode (n_groups > 0; launch_gemm_grouped): the problems share K.  Every 256x256 tile of every
    // problem is cut into `splits` runs of units_per_wg K slabs; unit u = split * total_tiles + tile leaves its
    // fp32 sums in slot u of `partial` ([slots][256][256]); reduce_grouped adds a tile's slots in split order.
    int n_groups, units_per_wg, slabs_per_tile, total_tiles;
    int max_units;        // grouped mode, in: if > 0, no more (tile, split) units than this unless one split exceeds it
    GemmGroup grp[kMaxGemmGroups];
    float* colsum;        // non-null (MFMA path only): column sums of C's values over bands of rows, fp32
                          // [bands][N]; band = colsum_row0 + 2 * (row tile) + (upper / lower half of the tile)
    int colsum_row0;
    Remap64 tbl;
    GemmRowSegments seg;  // launch_gemm_mfma_seg only
};

// launchers (defined in the kernel sources); each returns hipGetLastError()
// The next matrix-core launch (a GEMM of any form, or the attention backward) completes ev, as an event record behind
// it would, at less cost to its stream: the launch sites call take().  pending() tells whether a launch has taken
// it yet; next(nullptr) withdraws it.  One host thread per device at a time, like the calls themselves.
void launch_signal_next(hipEvent_t ev);
bool launch_signal_pending();
hipEvent_t launch_signal_take();
hipError_t launch_gemm_simple(const GemmArgs& g, int dtype, hipStream_t s);
// bf16 MFMA path; returns hipErrorNotSupported if the shape/strides do not fit it
hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s);
bool gemm_mfma_supported(const GemmArgs& g);
// C = A B (+ bias + residual) with A row-major, B's k through the remap table (REMAP_B_K) and K = positions of
// g.seg.slice columns of A: the tiles of a segment's rows walk only the positions set in its g.seg.pos (the
// caller guarantees that A is zero elsewhere, so the result is that of the full walk).  Takes g.seg.n, slice, end
// and pos; hipErrorNotSupported (nothing launched) if the shape does not fit.
hipError_t launch_gemm_mfma_kseg(const GemmArgs& g, hipStream_t s);
// The forms with A row-major (C = A B, no split-K, no residual) over row segments: prepare takes g->seg.n, slice,
// end and pos and fills the rest of g->seg, or returns hipErrorNotSupported if the shape does not fit (more than
// 64 tile rows or 16 tile columns of 256, K not a multiple of 64, operands the matrix-core path does not take);
// the launch takes a prepared g.
hipError_t gemm_mfma_seg_prepare(GemmArgs* g);
hipError_t launch_gemm_mfma_seg(const GemmArgs& g, hipStream_t s);
// Grouped weight-gradient launch (bf16 MFMA only).  The caller fills K, partial, n_groups and grp[].{A, B, lda,
// ldb, M, N}; the launcher fills the tile bookkeeping and returns it in *g for the reduction.  partial must hold
// gemm_grouped_slots(g) tiles of 256 x 256 floats.  hipErrorNotSupported if an operand does not fit the kernel.
size_t gemm_grouped_slots(const GemmArgs& g);
hipError_t launch_gemm_grouped(GemmArgs* g, hipStream_t s);
// out_g[r'][c'] (=|+=) sum over the slots of each tile, (r', c') through the group's remap
struct ReduceGroup {
    void* out;
    long ldo;
    int remap;      // RED_REMAP_*
    int table;      // which of the tables the remap uses
};
struct ReduceGroupedArgs {
    ReduceGroup grp[kMaxGemmGroups];
    Remap64 tbl[3];
};
hipError_t launch_reduce_grouped(int dtype, const GemmArgs& g, const ReduceGroupedArgs& r, int accumulate, hipStream_t s);
// rows of the output tile launch_gemm_mfma would pick (a tile makes two bands of g.colsum)
int gemm_mfma_tile_rows(const GemmArgs& g);
// static string naming the kernel instantiation launch_gemm_mfma would pick (for timing records)
const char* gemm_mfma_config_name(const GemmArgs& g);

hipError_t launch_ln_fwd(int dtype, const void* x, const void* gamma, const void* beta, void* y, float* mean,
                         float* rstd, int rows, int width, float eps, hipStream_t s);
// dx = LNbwd(d) + res
hipError_t launch_ln_bwd(int dtype, const void* d, const void* x, const float* mean, const float* rstd,
                         const void* gamma, const void* res, void* dx, int rows, int width, hipStream_t s);
// the same, also writing column sums of res (sum_res) and of dx (sum_out) over bands of rows:
// [ln_bwd_sums_bands(rows)][width] fp32 each; either may be null.  res must be given; width <= 2048.
bool ln_bwd_sums_supported(int width);
int ln_bwd_sums_bands(int rows);
hipError_t launch_ln_bwd_sums(int dtype, const void* d, const void* x, const float* mean, const float* rstd,
                              const void* gamma, const void* res, void* dx, int rows, int width, float* sum_res,
                              float* sum_out, hipStream_t s);
// partial_g/partial_b: [chunks][width] fp32 sums of d*xhat and d over row chunks
hipError_t launch_ln_param_grad(int dtype, const void* d, const void* x, const float* mean, const float* rstd,
                                float* partial_g, float* partial_b, int rows, int width, int chunks, hipStream_t s);
// partial: [chunks][cols] fp32 column sums over row chunks of X[rows][ld]
hipError_t launch_colsum(int dtype, const void* X, long ld, int rows, int cols, float* partial, int chunks,
                         hipStream_t s);

// RED_REMAP_F32 (grouped reduction only): the output is fp32, no remap, never accumulated
enum { RED_REMAP_NONE = 0, RED_REMAP_ROWS = 1, RED_REMAP_COLS = 2, RED_REMAP_F32 = 3 };
// out[r'][c'] (=|+=) scale * sum_s partial[s][r][c], (r',c') through the remap
hipError_t launch_reduce_partials(int dtype, const float* partial, int splits, long slice_stride, int rows, int cols,
                                  void* out, long ldo, int remap, const Remap64& tbl, int accumulate,
                                  hipStream_t s);

// per-head sums of squares (kind 0) or absolute values (kind 1) over the slices a head owns.
// A span is one slice family: for head h, elements p[first + h*head_stride + r*stride + c], r < rows,
// c < 8*cols8; it is worked on by nchunks workgroups (chunk0 = index of its first one).
// partial: [H][total_chunks] doubles, out: [H] doubles (both device)
struct ScoreSpan {
    const void* p;
    long first, head_stride, stride;
    int rows, cols8, chunk0, nchunks;
};
struct ScoreArgs {
    ScoreSpan span[16];
    int n, total_chunks, H;
};
hipError_t launch_subnet_scores(int dtype, const ScoreArgs& a, int kind, double* partial, double* out, hipStream_t s);

// the two subnets outside the blocks (kernels_head.hip)
hipError_t launch_im2col(int dtype, const void* img, void* patches, int B, int C, int H, int W, int P, hipStream_t s);
hipError_t launch_assemble_tokens(int dtype, const void* proj, const void* cls, const void* pos, void* tokens, int B, int Np,
                                  int D, hipStream_t s);
hipError_t launch_embed_bwd_gather(int dtype, const void* dtokens, void* dproj, void* g_pos, void* g_cls, int B, int Np, int D,
                                   int accumulate, hipStream_t s);
hipError_t launch_classifier(int dtype, const void* tokens, const void* ln_g, const void* ln_b, const void* w_c, const void* b_c,
                             const int32_t* labels, int B, int Tn, int D, int n, float eps, float* xhat, float* h, float* rstd,
                             float* logits, float* dl, float* loss_b, float* dh, void* dtokens, void* g_w_c, void* g_b_c,
                             void* g_ln_g, void* g_ln_b, float* loss, int accumulate, hipStream_t s);

// several independent column reductions out[c] = sum over chunks of partial[chunk][c] in one launch
// (the bias gradients of one block); remap_cols = 1 or 2 sends column c to tbl_a(c) or tbl_b(c)
struct ColReduceJob {
    const float* partial;
    void* out;
    int chunks, cols, remap_cols;
};
struct ColReduceBatch {
    ColReduceJob job[4];
    int n;
};
hipError_t launch_col_reduce_batch(int dtype, const ColReduceBatch& batch, const Remap64& tbl_a, const Remap64& tbl_b,
                                   int accumulate, hipStream_t s);


struct HeadList {
    int32_t n;
    uint8_t h[D2FT_MAX_HEADS];
};
// write +0.0 to every gradient slice of the listed heads (null pointers are skipped)
hipError_t launch_zero_head_slices(int dtype, const HeadList& heads, int H, int D, int r, void* g_wqkv, void* g_bqkv,
                                   void* g_wo, void* g_la_q, void* g_la_v, void* g_lb_q, void* g_lb_v,
                                   hipStream_t s);
// +0.0 into the feed-forward gradient slices (w1 rows, b1, w2 columns) of the listed heads; slice = Dm / H
hipError_t launch_zero_ffn_slices(int dtype, const HeadList& heads, int slice, int D, int Dm, void* g_w1, void* g_b1,
                                  void* g_w2, hipStream_t s);

// SGD with momentum over spans of tensors: for list entry y (blockIdx.y) the elements
// first + heads.h[y]*head_stride + r*stride + c, r < rows, c < 8*cols8, of w (storage dtype), g (storage
// dtype), v (fp32) and, if non-NULL, master (fp32)
struct SgdSpan {
    void* w;
    const void* g;
    float* v;
    float* master;
    long first, head_stride, stride;
    int rows, cols8, chunk0, nchunks;
};
struct SgdArgs {
    SgdSpan span[16];
    int n, total_chunks;
    float lr, momentum, weight_decay;
};
hipError_t launch_sgd(int dtype, const SgdArgs& a, const HeadList& heads, hipStream_t s);


// W_eff rows for compacted heads: out[(j*3+p)*64 + d][:] = W[p][live[j]][d][:] (+ s * B A for p in {query, value})
hipError_t launch_lora_merge(int dtype, const void* w_qkv, const void* la_q, const void* la_v, const void* lb_q,
                             const void* lb_v, void* out, const HeadList& live, int n_heads_used, int H, int D, int r,
                             float scale, hipStream_t s);
// LoRA gradients from G = dW_eff (fp32, compacted rows as in launch_lora_merge, split-K slices summed here):
//   dB[h] (=|+=) s * G_h A_h^T,  dA[h] (=|+=) s * B_h^T G_h   for the query and value planes
hipError_t launch_lora_project(int dtype, const float* G, int splits, long slice_stride, const void* la_q,
                               const void* la_v, const void* lb_q, const void* lb_v, void* g_la_q, void* g_la_v,
                               void* g_lb_q, void* g_lb_v, const HeadList& full, int H, int D, int r, float scale,
                               int accumulate, hipStream_t s);

// attention over compacted heads.  qkv: [rows][ldq], head j at columns j*192 (+0 Q, +64 K, +128 V);
// o: [rows][ldo], head j at columns j*64; lse: [n_full][rows] (written for j < n_full only)
hipError_t launch_attn_fwd_simple(int dtype, const void* qkv, long ldq, void* o, long ldo, float* lse, int batch,
                                  int tokens, int n_live, int n_full, hipStream_t s);
// d_o: [rows][ld_do] head j at j*64; dqkv: [rows][ld_dqkv] head j at j*192; delta: [n_full][rows] scratch
hipError_t launch_attn_bwd_simple(int dtype, const void* qkv, long ldq, const void* o, long ldo, const float* lse,
                                  const void* d_o, long ld_do, void* dqkv, long ld_dqkv, float* delta, int batch,
                                  int tokens, int n_full, hipStream_t s);

// MFMA attention (bf16, head dimension 64, up to 256 tokens forward, 224 backward); same argument meaning as the simple launchers
// Which (micro-batch, compacted head position) pairs take part when one launch covers several
// micro-batches with their own op codes: bit p of live[i] / full[i] says whether the head at position p
// is computed / is p_f in micro-batch i, which holds the images [img_end[i-1], img_end[i]).
struct MicroMask {
    int n;
    int n_live_pos, n_full_pos;   // positions of the union layout: live ones, and its p_f prefix
    int img_end[D2FT_MAX_MICRO];
    uint64_t live[D2FT_MAX_MICRO];
    uint64_t full[D2FT_MAX_MICRO];
    __host__ __device__ int micro_of(int image) const {
        int i = 0;
        while (i + 1 < n && image >= img_end[i]) ++i;
        return i;
    }
};

bool attn_mfma_supported(int tokens, long ldq, long ldo);       // forward: up to 256 tokens
bool attn_bwd_mfma_supported(int tokens, long ldq, long ldo);   // backward: up to 224 tokens
// with a mask: pairs that are not live get a zero O block (forward), pairs that are not p_f a zero dQKV
// block (backward); the log-sum-exp is saved for p_f pairs.  The grid has one workgroup per image and
// "slot" (as many slots as the busiest micro-batch has pairs that take part): slot s of an image works
// on its micro-batch's s-th such pair, and the zero blocks are dealt round-robin over the slots, so no
// workgroup exists only to write zeros.
hipError_t launch_attn_fwd_mfma_masked(const void* qkv, long ldq, void* o, long ldo, float* lse, int batch, int tokens,
                                       int n_live, const MicroMask& mask, hipStream_t s);
hipError_t launch_attn_bwd_mfma_masked(const void* qkv, long ldq, const void* o, long ldo, const float* lse,
                                       const void* d_o, long ld_do, void* dqkv, long ld_dqkv, float* bsum, long ld_bsum,
                                       int batch, int tokens, int n_full, const MicroMask& mask, hipStream_t s);
// zero the [tokens][width] blocks (column offset position * width, row stride ld; in x and, if given, x2) of
// the pairs at positions 0 .. n_pos-1 that are skipped, or that are live but not p_f
enum { PAIRS_SKIPPED = 0, PAIRS_FORWARD_ONLY = 1 };
hipError_t launch_zero_pairs(int dtype, void* x, void* x2, long ld, int batch, int tokens, int n_pos, int width, int which,
                             const MicroMask& mask, hipStream_t s);
hipError_t launch_attn_fwd_mfma(const void* qkv, long ldq, void* o, long ldo, float* lse, int batch, int tokens,
                                int n_live, int n_full, hipStream_t s);
// bsum: null, or [batch][ld_bsum] fp32: row b receives the column sums of image b's dqkv rows (the first
// n_full * 192 columns), i.e. partial sums of the QKV bias gradient
hipError_t launch_attn_bwd_mfma(const void* qkv, long ldq, const void* o, long ldo, const float* lse,
                                const void* d_o, long ld_do, void* dqkv, long ld_dqkv, float* bsum, long ld_bsum,
                                int batch, int tokens, int n_full, hipStream_t s);

// bi-level knapsack (Alg. 1 + Alg. 2); all pointers are device pointers into the caller's workspace
struct KnapsackArgs {
    int n_knapsacks, n_items;
    const double* score_full;   // [K][n]
    const double* score_fwd;    // [K][n]
    const int* cost_fwd;        // [K]
    const int* cost_bwd;        // [K]
    const int* cap_full;        // [K]
    const int* cap_fwd;         // [K]
    double* rows;               // [K*2 problems][2][stride]   two rows of the DP value table
    uint8_t* changed;           // [K*2 problems][n][stride]   T[i][w] != T[i-1][w]
    uint8_t* selected;          // [K*2 problems][n]           0/1 tables of the two stages
    long stride;                // max capacity + 1, rounded up
};
hipError_t launch_knapsack(const KnapsackArgs& a, uint8_t* ops_dev, hipStream_t s);

}  // namespace d2ft
