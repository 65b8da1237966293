// C ABI entry points of libd2ft: argument validation, head compaction, buffer layout and the
// launch sequence of one block's forward and backward pass.  All device work is in the
// kernels_*.hip files; nothing here allocates device memory or keeps state between calls.
#include <math.h>
#include <string.h>

#include <map>
#include <string>
#include <vector>

#include "d2ft_common.h"

namespace d2ft {

namespace {

constexpr int kMaxSplits = 8;
constexpr int kColChunks = 64;

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline size_t elem_size(int dtype) { return dtype == D2FT_F32 ? 4 : 2; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Dims {
    int B, T, D, H, Dm, r;
    long M;
    int dtype;
    size_t es;
};

bool desc_ok(const d2ft_block_desc* d, d2ft_status* why) {
    if (!d) { *why = D2FT_EINVAL; return false; }
    if (d->dtype != D2FT_F32 && d->dtype != D2FT_BF16) { *why = D2FT_EINVAL; return false; }
    if (!(d->ln_eps > 0.0f) || !isfinite(d->ln_eps) || !isfinite(d->lora_scale)) { *why = D2FT_EINVAL; return false; }
    *why = D2FT_ESHAPE;
    if (d->batch < 1 || d->tokens < 1 || d->tokens > 1024) return false;
    if (d->width < 8 || d->width % 8) return false;
    if (d->mlp_hidden < 8 || d->mlp_hidden % 8) return false;
    if (d->heads < 1 || d->heads > D2FT_MAX_HEADS) return false;
    if (d->head_dim != D2FT_HEAD_DIM) return false;
    if (d->lora_rank < 0 || d->lora_rank > D2FT_MAX_LORA_RANK) return false;
    if ((long)d->batch * d->tokens > (1L << 24)) return false;
    if (d->flags & D2FT_FLAG_GATE_FFN) {   // a head's feed-forward slice is a whole number of 64-column blocks
        if (d->mlp_hidden % d->heads) return false;
        const int slice = d->mlp_hidden / d->heads;
        if (slice % 64 || d->mlp_hidden / 64 > kMaxBlocks64) return false;
    }
    *why = D2FT_OK;
    return true;
}

Dims dims_of(const d2ft_block_desc* d) {
    Dims s;
    s.B = d->batch; s.T = d->tokens; s.D = d->width; s.H = d->heads; s.Dm = d->mlp_hidden; s.r = d->lora_rank;
    s.M = (long)d->batch * d->tokens;
    s.dtype = d->dtype;
    s.es = elem_size(d->dtype);
    return s;
}

// ---- layout of the saved buffer (forward -> backward) ----
struct SavedLayout {
    size_t mean1, rstd1, u, qkv, o, lse, x1, mean2, rstd2, v, z, g, weff, total;
};
SavedLayout saved_layout(const Dims& s) {
    SavedLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off += align256(bytes); return at; };
    L.mean1 = take(s.M * 4);
    L.rstd1 = take(s.M * 4);
    L.u = take(s.M * s.D * s.es);
    L.qkv = take(s.M * s.H * 192 * s.es);
    L.o = take(s.M * s.H * 64 * s.es);
    L.lse = take((size_t)s.H * s.M * 4);
    L.x1 = take(s.M * s.D * s.es);
    L.mean2 = take(s.M * 4);
    L.rstd2 = take(s.M * 4);
    L.v = take(s.M * s.D * s.es);
    L.z = take(s.M * s.Dm * s.es);   // GELU'(z) of the hidden units in use (what the backward needs of z)
    L.g = take(s.M * s.Dm * s.es);
    // LoRA: the merged QKV weights of the live heads (compacted order), built by the forward call and read
    // again by the backward call (the p_f heads are the first rows)
    L.weff = take(s.r > 0 ? (size_t)192 * s.H * s.D * s.es : 0);
    L.total = off;
    return L;
}

// ---- layout of the scratch buffer ----
struct ScratchLayout {
    size_t part, colpart, colfuse_b1, colfuse_b2, colfuse_bo, colfuse_bqkv, colfuse_set, dz, dz_alt, dv, dx1, d_o, dqkv, du, delta, lora_g, total;
    size_t part_floats, colpart_stride;
};
ScratchLayout scratch_layout(const Dims& s) {
    ScratchLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off += align256(bytes); return at; };
    size_t mat = (size_t)s.Dm * s.D;
    if ((size_t)192 * s.H * s.D > mat) mat = (size_t)192 * s.H * s.D;
    size_t cols = s.Dm;
    if ((size_t)192 * s.H > cols) cols = 192 * s.H;
    if ((size_t)s.D > cols) cols = s.D;
    L.part_floats = mat * kMaxSplits;
    {   // or one 256 x 256 tile per (workgroup, tile) pair of the grouped weight-gradient launch
        auto t256 = [](size_t r, size_t c) { return ((r + 255) / 256) * ((c + 255) / 256); };
        const size_t tiles = 2 * t256(s.Dm, s.D) + t256(s.D, (size_t)64 * s.H) + t256((size_t)192 * s.H, s.D);
        const size_t grouped = tiles * 8 * 65536;   // up to 8 splits
        if (grouped > L.part_floats) L.part_floats = grouped;
    }
    L.part = take(L.part_floats * 4);
    L.colpart_stride = (size_t)kColChunks * cols;   // floats per region: four bias reductions, two LayerNorm ones
    L.colpart = take(6 * L.colpart_stride * 4);
    // column sums that the producing kernels write themselves, one row of partial sums per band of rows:
    // the dz GEMM's epilogue (bands of 64 or more rows) for b1, the LayerNorm backward for b2 and b_o
    L.colfuse_b1 = take(((size_t)s.M / 64 + 8) * s.Dm * 4);
    L.colfuse_b2 = take((size_t)ln_bwd_sums_bands((int)s.M) * s.D * 4);
    L.colfuse_bo = take((size_t)ln_bwd_sums_bands((int)s.M) * s.D * 4);
    L.colfuse_bqkv = take((size_t)s.B * s.H * 192 * 4);   // per image, from the attention backward
    // and a second set of the four: consecutive backward calls alternate, so that a call may write its sums
    // while the reduction of the call before, left on the side stream (D2FT_FLAG_DEFER_JOIN), still reads its own
    L.colfuse_set = take(0) - L.colfuse_b1;
    take(L.colfuse_set);
    L.dz = take(s.M * s.Dm * s.es);
    L.dz_alt = take(s.M * s.Dm * s.es) - L.dz;   // consecutive backward calls alternate (as for the column sums above)
    L.dv = take(s.M * s.D * s.es);
    L.dx1 = take(s.M * s.D * s.es);
    L.d_o = take(s.M * s.H * 64 * s.es);
    L.dqkv = take(s.M * s.H * 192 * s.es);
    L.du = take(s.M * s.D * s.es);
    L.delta = take((size_t)s.H * s.M * 4);
    L.lora_g = take(s.r > 0 ? (size_t)192 * s.H * s.D * 4 : 0);   // fp32 dW_eff of the p_f heads, for the LoRA gradients
    L.total = off;
    return L;
}

d2ft_status compact(const uint8_t* ops, int heads, int32_t* live, int32_t* n_full, int32_t* n_live) {
    if (!ops || !live || !n_full || !n_live) return D2FT_EINVAL;
    if (heads < 1 || heads > D2FT_MAX_HEADS) return D2FT_ESHAPE;
    int nf = 0, nl = 0;
    for (int h = 0; h < heads; ++h) {
        if (ops[h] != D2FT_OP_FULL && ops[h] != D2FT_OP_FWD && ops[h] != D2FT_OP_SKIP) return D2FT_EINVAL;
    }
    for (int h = 0; h < heads; ++h)
        if (ops[h] == D2FT_OP_FULL) live[nl++] = h;
    nf = nl;
    for (int h = 0; h < heads; ++h)
        if (ops[h] == D2FT_OP_FWD) live[nl++] = h;
    *n_full = nf;
    *n_live = nl;
    return D2FT_OK;
}

bool weights_ok(const d2ft_block_desc* d, const d2ft_block_weights* w) {
    if (!w) return false;
    const void* req[] = {w->ln1_g, w->ln1_b, w->w_qkv, w->b_qkv, w->w_o, w->ln2_g, w->ln2_b, w->w1, w->b1, w->w2};
    for (const void* p : req)
        if (!p || !aligned16(p)) return false;
    if ((w->b_o && !aligned16(w->b_o)) || (w->b2 && !aligned16(w->b2))) return false;
    if (d->lora_rank > 0) {
        const void* lo[] = {w->lora_a_q, w->lora_a_v, w->lora_b_q, w->lora_b_v};
        for (const void* p : lo)
            if (!p || !aligned16(p)) return false;
    }
    return true;
}

// compacted-QKV remap: 64-row block j*3+p of the compacted weight is plane p, head live[j]
void fill_qkv_table(Remap64& t, const int32_t* live, int n, int H) {
    for (int j = 0; j < n; ++j)
        for (int p = 0; p < 3; ++p) t.start[j * 3 + p] = (p * H + live[j]) * 64;
}
void fill_head_table(Remap64& t, const int32_t* live, int n) {
    for (int j = 0; j < n; ++j) t.start[j] = live[j] * 64;
}
// hidden units of the feed-forward slices of the first n listed heads, slice = Dm / H (a multiple of 64)
void fill_ffn_table(Remap64& t, const int32_t* live, int n, int slice) {
    const int per = slice / 64;
    for (int j = 0; j < n; ++j)
        for (int b = 0; b < per; ++b) t.start[j * per + b] = live[j] * slice + b * 64;
}

// ---- optional per-kernel timing (diagnostics; see d2ft_timing_enable in d2ft.h) ----
struct TimingRec {
    std::string label;
    double flops, bytes;
    hipEvent_t a, b;
};
struct TimingState {
    bool on = false;
    std::vector<TimingRec> recs;
    std::vector<hipEvent_t> pool;
    const char* label = nullptr;   // set by a launcher wrapper to refine the class of the next record
    double flops = 0, bytes = 0;
    bool open = false;
};
TimingState g_timing;
constexpr size_t kMaxTimingRecs = 100000;

hipEvent_t timing_event() {
    if (!g_timing.pool.empty()) {
        hipEvent_t e = g_timing.pool.back();
        g_timing.pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void timing_begin(hipStream_t st, const char* what) {
    g_timing.open = false;
    if (!g_timing.on || g_timing.recs.size() >= kMaxTimingRecs) return;
    TimingRec r;
    const char* paren = strchr(what, '(');
    r.label = paren ? std::string(what, paren - what) : std::string(what);
    r.flops = r.bytes = 0;
    r.a = timing_event();
    r.b = timing_event();
    if (!r.a || !r.b) return;
    g_timing.label = nullptr;
    g_timing.flops = g_timing.bytes = 0;
    if (hipEventRecord(r.a, st) != hipSuccess) return;
    g_timing.recs.push_back(r);
    g_timing.open = true;
}

void timing_end(hipStream_t st) {
    if (!g_timing.open) return;
    TimingRec& r = g_timing.recs.back();
    (void)hipEventRecord(r.b, st);
    if (g_timing.label) r.label = g_timing.label;
    r.flops = g_timing.flops;
    r.bytes = g_timing.bytes;
    g_timing.open = false;
}

#define D2FT_TRY_UNTIMED(expr)                      \
    do {                                            \
        hipError_t e__ = (expr);                    \
        if (e__ != hipSuccess) return D2FT_EDEVICE; \
    } while (0)

// every launch site has the stream in a variable called st
#define D2FT_TRY(expr)                              \
    do {                                            \
        timing_begin(st, #expr);                    \
        hipError_t e__ = (expr);                    \
        timing_end(st);                             \
        if (e__ != hipSuccess) return D2FT_EDEVICE; \
    } while (0)

// a bandwidth-bound launch: also books the algorithmic bytes it moves (read + written once each)
#define D2FT_TRY_BYTES(nbytes, expr)                \
    do {                                            \
        timing_begin(st, #expr);                    \
        hipError_t e__ = (expr);                    \
        g_timing.bytes = (double)(nbytes);          \
        timing_end(st);                             \
        if (e__ != hipSuccess) return D2FT_EDEVICE; \
    } while (0)

// the event that this thread's next matrix-core launch is to complete (launch_signal_next)
thread_local hipEvent_t g_launch_signal = nullptr;

// one timed GEMM launch (the launch sites use D2FT_TRY_UNTIMED around run_gemm)
hipError_t timed_mfma(const GemmArgs& g, hipStream_t st, hipEvent_t done = nullptr) {
    if (done) launch_signal_next(done);
    timing_begin(st, "gemm");
    g_timing.label = gemm_mfma_config_name(g);
    g_timing.flops = 2.0 * g.M * g.N * g.K;
    const hipError_t e = launch_gemm_mfma(g, st);
    timing_end(st);
    return e;
}

// true if run_gemm takes the matrix-core path for g (the only path that honours g.colsum)
bool on_mfma_path(const GemmArgs& g, const d2ft_block_desc* d) {
    return d->dtype == D2FT_BF16 && !(d->flags & D2FT_FLAG_NO_MFMA) && gemm_mfma_supported(g);
}

// colsum_bands: if non-null, receives the number of rows of g.colsum the launches fill
// done: if non-null, the call's last matrix-core launch completes it (gemm_mfma_signal_next); the caller checks
// launch_signal_pending() for the paths that have no such launch
hipError_t run_gemm(const GemmArgs& g, const d2ft_block_desc* d, hipStream_t s, int* colsum_bands = nullptr,
                    hipEvent_t done = nullptr) {
    if (colsum_bands) *colsum_bands = 0;
    if (on_mfma_path(g, d)) {
        // Tile plan for shapes of more than one round of the chip's 256 CUs.  The one-per-CU tiles take whole
        // rounds however few tiles the last one has, so three plans are priced in microseconds with per-round
        // costs measured on this part (a round = fixed cost + slabs of 64 of K; ep = the epilogue's extra work):
        // all 256x256 tiles; the rows of the whole rounds as 256x256 tiles and the remaining rows as 128x128
        // tiles, two of which share a CU; all 192x256 tiles.
        if (!g.partial && g.tile_hint == 0 && g.M >= 512 && g.N >= 256) {
            const long tn = (g.N + 255) / 256, tm = (g.M + 255) / 256, total = tm * tn;
            const double slabs = (g.K + 63) / 64;
            const double ep = g.act == ACT_GELU ? 8.0 : ((g.act == ACT_DGELU || g.residual) ? 3.0 : 0.0);
            auto rounds_of = [](long tiles, long per_round) { return (double)((tiles + per_round - 1) / per_round); };
            const double r256 = 8.5 + 1.6 * slabs + ep, r192 = 9.0 + 1.1 * slabs + 0.75 * ep, r128 = 8.0 + 1.2 * slabs + 0.4 * ep;
            if (total > 256) {
                const double c_all256 = rounds_of(total, 256) * r256;
                const double c_all192 = rounds_of((long)((g.M + 191) / 192) * tn, 256) * r192;
                const long rounds = total / 256;
                const long tm_big = rounds * 256 / tn;
                const long m_split = tm_big * 256;
                double c_split = 1e30;
                if (m_split > 0 && m_split < g.M) {
                    const long rest_tiles = ((g.M - m_split + 127) / 128) * ((g.N + 127) / 128);
                    c_split = rounds_of(tm_big * tn, 256) * r256 + rounds_of(rest_tiles, 512) * r128;
                }
                if (c_split < c_all256 && c_split < c_all192) {
                    GemmArgs big = g, rest = g;
                    big.M = (int)m_split;
                    big.tile_hint = 1;
                    rest.M = g.M - (int)m_split;
                    rest.tile_hint = 2;
                    const size_t es = 2;
                    rest.A = static_cast<const char*>(g.A) + m_split * g.a_rs * es;
                    rest.C = static_cast<char*>(g.C) + m_split * g.ldc * es;
                    if (g.residual) rest.residual = static_cast<const char*>(g.residual) + m_split * g.ldr * es;
                    if (g.Z) rest.Z = static_cast<char*>(g.Z) + m_split * g.ldz * es;
                    rest.colsum_row0 = g.colsum_row0 + 2 * (int)tm_big;
                    if (gemm_mfma_supported(big) && gemm_mfma_supported(rest)) {
                        if (colsum_bands) *colsum_bands = 2 * (int)tm_big + 2 * ((rest.M + 127) / 128);
                        hipError_t e = timed_mfma(big, s);
                        if (e != hipSuccess) return e;
                        return timed_mfma(rest, s, done);
                    }
                } else if (c_all192 < c_all256) {
                    GemmArgs t = g;
                    t.tile_hint = 3;
                    if (gemm_mfma_supported(t)) {
                        if (colsum_bands) *colsum_bands = 2 * ((g.M + 191) / 192);
                        return timed_mfma(t, s, done);
                    }
                }
            }
        }
        if (colsum_bands) {
            const int bm = gemm_mfma_tile_rows(g);
            *colsum_bands = 2 * ((g.M + bm - 1) / bm);
        }
        return timed_mfma(g, s, done);
    }
    if (g.colsum) return hipErrorNotSupported;   // callers ask on_mfma_path() first
    timing_begin(s, "gemm");
    g_timing.label = "gemm_simple_kernel";
    g_timing.flops = 2.0 * g.M * g.N * g.K;
    const hipError_t e = launch_gemm_simple(g, d->dtype, s);
    timing_end(s);
    return e;
}

// A gated feed-forward product over the whole batch whose micro-batches have their own codes: the rows of
// micro-batch i times the slices (positions of `slice` columns) in pos_of[i], zeros elsewhere; 256x256 tiles
// that no micro-batch needs are not multiplied.  hipErrorNotSupported (nothing launched) if the shape does not
// fit: the caller then multiplies the union of the slices over all rows and zeroes afterwards.
hipError_t run_gemm_segments(GemmArgs g, const d2ft_block_desc* d, const MicroMask& mask, const uint64_t* pos_of, int tokens,
                             int slice, hipStream_t s, int* colsum_bands = nullptr, hipEvent_t done = nullptr) {
    if (colsum_bands) *colsum_bands = 0;
    if (!on_mfma_path(g, d) || mask.n > kMaxGemmSegments) return hipErrorNotSupported;
    g.seg.n = mask.n;
    g.seg.slice = slice;
    double cols = 0.0;   // row x column pairs that take part
    for (int i = 0; i < mask.n; ++i) {
        g.seg.end[i] = mask.img_end[i] * tokens;
        g.seg.pos[i] = pos_of[i];
        cols += (double)(mask.img_end[i] - (i ? mask.img_end[i - 1] : 0)) * tokens * __builtin_popcountll(pos_of[i]) * slice;
    }
    if (gemm_mfma_seg_prepare(&g) != hipSuccess) return hipErrorNotSupported;
    if (colsum_bands) *colsum_bands = 2 * ((g.M + 255) / 256);
    if (done) launch_signal_next(done);
    timing_begin(s, "gemm");
    g_timing.label = g.b_rs != 1 ? "gemm_mfma_kernel<256, 256, 64, 2, 4, false, true, 1, false, false, true, 1>"
                                 : "gemm_mfma_kernel<256, 256, 64, 2, 4, false, false, 1, false, false, true, 0>";
    g_timing.flops = 2.0 * cols * g.K;
    const hipError_t e = launch_gemm_mfma_seg(g, s);
    timing_end(s);
    return e;
}

// A product whose K index runs over the gated slices (FC2 forward, the backward's dv) or over the heads (output
// projection forward, the backward's du) while the micro-batches have their own codes: A's columns of a slice are
// zero in the rows of a micro-batch in which the slice does not take part (pos_of[i]: the slices of micro-batch
// i), so every tile walks only the slices of its own micro-batch.  The sums are those of the full walk.  hipErrorNotSupported (nothing launched) if the shape does not fit.
hipError_t run_gemm_kseg(GemmArgs g, const d2ft_block_desc* d, const MicroMask& mask, const uint64_t* pos_of, int tokens,
                         int slice, hipStream_t s) {
    if (!on_mfma_path(g, d) || mask.n > kMaxGemmSegments) return hipErrorNotSupported;
    g.seg.n = mask.n;
    g.seg.slice = slice;
    double ks = 0.0;   // row x k pairs that are walked if no tile straddles two micro-batches
    for (int i = 0; i < kMaxGemmSegments; ++i) {
        g.seg.end[i] = i < mask.n ? mask.img_end[i] * tokens : g.M;
        g.seg.pos[i] = i < mask.n ? pos_of[i] : 0;
        if (i < mask.n) ks += (double)(mask.img_end[i] - (i ? mask.img_end[i - 1] : 0)) * tokens * __builtin_popcountll(pos_of[i]) * slice;
    }
    timing_begin(s, "gemm");
    if (g_timing.on) {
        static char label[160];
        snprintf(label, sizeof(label), "%s k-segments", gemm_mfma_config_name(g));
        g_timing.label = label;
        g_timing.flops = 2.0 * ks * g.N;
    }
    const hipError_t e = launch_gemm_mfma_kseg(g, s);
    timing_end(s);
    return e;
}

// bf16, head dimension 64, up to 224 tokens: the matrix-core attention kernels, forward and backward
static bool attn_on_mfma(const d2ft_block_desc* d) {
    return d->dtype == D2FT_BF16 && !(d->flags & D2FT_FLAG_NO_MFMA) && d->tokens <= 224;
}

hipError_t run_attn_fwd(const d2ft_block_desc* d, const void* qkv, long ldq, void* o, long ldo, float* lse, int batch,
                        int tokens, int n_live, int n_full, hipStream_t s, const MicroMask* mask = nullptr) {
    g_timing.flops = 4.0 * batch * n_live * (double)tokens * tokens * 64;
    if (mask) {   // callers pass a mask only where attn_on_mfma() holds
        g_timing.label = "attn_fwd_mfma";
        return launch_attn_fwd_mfma_masked(qkv, ldq, o, ldo, lse, batch, tokens, n_live, *mask, s);
    }
    if (d->dtype == D2FT_BF16 && !(d->flags & D2FT_FLAG_NO_MFMA) && attn_mfma_supported(tokens, ldq, ldo)) {
        g_timing.label = "attn_fwd_mfma";
        return launch_attn_fwd_mfma(qkv, ldq, o, ldo, lse, batch, tokens, n_live, n_full, s);
    }
    g_timing.label = "attn_fwd_simple";
    return launch_attn_fwd_simple(d->dtype, qkv, ldq, o, ldo, lse, batch, tokens, n_live, n_full, s);
}

// the matrix-core backward also sums the columns of dqkv per image (bsum, see launch_attn_bwd_mfma)
static bool attn_bwd_on_mfma(const d2ft_block_desc* d, int tokens, long ldq, long ldo, long ld_do, long ld_dqkv) {
    return d->dtype == D2FT_BF16 && !(d->flags & D2FT_FLAG_NO_MFMA) && attn_bwd_mfma_supported(tokens, ldq, ldo) &&
           (ld_do % 8) == 0 && (ld_dqkv % 8) == 0;
}

// done: if non-null, the matrix-core launch completes it (the caller checks launch_signal_pending() for the path
// that has none)
hipError_t run_attn_bwd(const d2ft_block_desc* d, const void* qkv, long ldq, const void* o, long ldo, const float* lse,
                        const void* d_o, long ld_do, void* dqkv, long ld_dqkv, float* delta, float* bsum, int batch,
                        int tokens, int n_full, hipStream_t s, const MicroMask* mask = nullptr, hipEvent_t done = nullptr) {
    if (done) launch_signal_next(done);
    g_timing.flops = 8.0 * batch * n_full * (double)tokens * tokens * 64;
    if (mask) {
        g_timing.label = "attn_bwd_mfma";
        return launch_attn_bwd_mfma_masked(qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv, ld_dqkv, bsum, ld_dqkv, batch, tokens,
                                           n_full, *mask, s);
    }
    if (attn_bwd_on_mfma(d, tokens, ldq, ldo, ld_do, ld_dqkv)) {
        g_timing.label = "attn_bwd_mfma";
        return launch_attn_bwd_mfma(qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv, ld_dqkv, bsum, ld_dqkv, batch, tokens, n_full, s);
    }
    if (bsum) return hipErrorNotSupported;   // callers ask attn_bwd_on_mfma() first
    g_timing.label = "attn_bwd_simple";
    return launch_attn_bwd_simple(d->dtype, qkv, ldq, o, ldo, lse, d_o, ld_do, dqkv, ld_dqkv, delta, batch, tokens, n_full,
                                  s);
}

GemmArgs gemm_base() {
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.splits = 1;
    return g;
}

// Split count and tile of a weight-gradient GEMM (reduction over the token rows).  The 256x256 tile
// runs one workgroup per CU, so the splits should bring the grid close to, but not above, the 256
// CUs; outputs too small for that use the 128x128 tile, of which two fit a CU.
int pick_splits(long out_rows, long out_cols, long K, int* tile_hint) {
    const long t256 = ((out_rows + 255) / 256) * ((out_cols + 255) / 256);
    const long t128 = ((out_rows + 127) / 128) * ((out_cols + 127) / 128);
    long s;
    if (t256 >= 24 && out_rows >= 256 && out_cols >= 256) {
        *tile_hint = 1;
        s = 256 / t256;
    } else {
        *tile_hint = 2;
        s = 512 / t128;
    }
    if (s > kMaxSplits) s = kMaxSplits;
    while (s > 1 && K / s < 512) --s;
    return s < 1 ? 1 : (int)s;
}

int pick_chunks(long rows) {
    long c = rows / 64;
    if (c < 1) c = 1;
    if (c > kColChunks) c = kColChunks;
    return (int)c;
}

// weight gradient dW[out_rows][out_cols] = Aop^T Bop over the token rows, reduced through fp32 partials
//   Aop: [M][lda] columns a_col0.. (out_rows of them), Bop: [M][ldb] columns (out_cols of them)
d2ft_status weight_grad(const d2ft_block_desc* d, const Dims& s, const void* Aop, long lda, const void* Bop, long ldb,
                        int out_rows, int out_cols, float* part, void* out, long ldo, int red_remap,
                        const Remap64& tbl, hipStream_t st, int* splits_out = nullptr, bool reduce = true) {
    GemmArgs g = gemm_base();
    g.A = Aop; g.a_rs = 1; g.a_cs = lda;      // A(m = out row, k = token) = Aop[token][m]
    g.B = Bop; g.b_rs = ldb; g.b_cs = 1;      // B(k = token, n = out col) = Bop[token][n]
    g.M = out_rows; g.N = out_cols; g.K = (int)s.M;
    g.partial = part;
    g.splits = pick_splits(out_rows, out_cols, s.M, &g.tile_hint);
    if (splits_out) *splits_out = g.splits;
    D2FT_TRY_UNTIMED(run_gemm(g, d, st));
    if (reduce)
        D2FT_TRY_BYTES((4.0 * g.splits + s.es) * out_rows * out_cols, launch_reduce_partials(s.dtype, part, g.splits, (long)out_rows * out_cols, out_rows, out_cols, out,
                                        ldo, red_remap, tbl, (d->flags & D2FT_FLAG_ACCUM_GRADS) ? 1 : 0, st));
    return D2FT_OK;
}

// The weight gradients of one backward call, collected and run as ONE grouped launch at the end of the call:
// each is a reduction over the token rows, and together they have enough tiles to fill the chip with about a
// third of the split-K partial traffic that separate launches need.
struct WeightGradBatch {
    bool enabled;
    GemmArgs g;
    ReduceGroupedArgs r;
    // a group with remap RED_REMAP_F32 leaves its fp32 product for a consumer: after the flush f32_splits says
    // how (0: summed, in the group's out; n > 0: n split-K slices, one after the other, at the start of `part`)
    int f32_splits;
};

void weight_grad_batch_init(WeightGradBatch* b, const d2ft_block_desc* d) {
    memset(b, 0, sizeof(*b));
    b->g.splits = 1;
    b->enabled = d->dtype == D2FT_BF16 && !(d->flags & D2FT_FLAG_NO_MFMA);
}

// queue dW[out_rows][out_cols] = Aop^T Bop (arguments as weight_grad); table_slot: which of the batch's three
// remap tables tbl is kept in
d2ft_status weight_grad_queue(WeightGradBatch* b, const d2ft_block_desc* d, const Dims& s, const void* Aop, long lda,
                              const void* Bop, long ldb, int out_rows, int out_cols, float* part, void* out, long ldo,
                              int red_remap, const Remap64& tbl, int table_slot, hipStream_t st) {
    if (!b->enabled || b->g.n_groups >= kMaxGemmGroups)
        return weight_grad(d, s, Aop, lda, Bop, ldb, out_rows, out_cols, part, out, ldo, red_remap, tbl, st);
    const int i = b->g.n_groups++;
    GemmGroup& G = b->g.grp[i];
    G.A = Aop; G.lda = lda; G.B = Bop; G.ldb = ldb; G.M = out_rows; G.N = out_cols;
    ReduceGroup& R = b->r.grp[i];
    R.out = out; R.ldo = ldo; R.remap = red_remap; R.table = table_slot;
    b->r.tbl[table_slot] = tbl;
    return D2FT_OK;
}

// A second stream of the library's own, per device, with the two events that order it against the caller's
// stream.  A backward call puts the weight-gradient launches with their reductions on it - nothing else in the
// call waits for them - so that they run beside the chain of launches that leads to dx, most of which leave CUs
// idle (GEMMs of fewer tiles than CUs, partial last rounds, the attention backward).  Default priority; a call
// ends joined, so that to the caller the whole call is work on its own stream, unless the caller hands the join
// on with D2FT_FLAG_DEFER_JOIN.  `fork` is recorded on the caller's stream, or completed by the launch the side
// stream has to wait for (launch_signal_next), and waited for by the side stream; `join` the other way round.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool failed = false;
    // D2FT_FLAG_DEFER_JOIN: a call has returned with work still on the stream (`join` marks its end).
    // pending_dims: the call's shape, i.e. its scratch layout.
    bool pending = false;
    Dims pending_dims;
    int parity = 0;   // which set of fused column-sum regions the last backward call used
};
// the current device's side stream; create = false: only if it exists already
SideStream* side_stream(bool create = true) {
    static SideStream per_device[16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
    SideStream& S = per_device[dev];
    if (S.failed) return nullptr;
    if (!S.stream) {
        if (!create) return nullptr;
        if (hipStreamCreateWithFlags(&S.stream, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&S.fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&S.join, hipEventDisableTiming) != hipSuccess) {
            S.failed = true;
            S.stream = nullptr;
            return nullptr;
        }
    }
    return &S;
}
// Orders st behind whatever an earlier call with D2FT_FLAG_DEFER_JOIN left running on the side stream.  Every
// entry point that launches work starts with it (the backward takes a cheaper route of its own when it can).
d2ft_status join_pending(hipStream_t st) {
    SideStream* S = side_stream(false);
    if (!S || !S->pending) return D2FT_OK;
    S->pending = false;
    return hipStreamWaitEvent(st, S->join, 0) == hipSuccess ? D2FT_OK : D2FT_EDEVICE;
}
// work launched on S->stream from here on starts after what `st` holds now
bool side_fork(SideStream* S, hipStream_t st) {
    return hipEventRecord(S->fork, st) == hipSuccess && hipStreamWaitEvent(S->stream, S->fork, 0) == hipSuccess;
}

// part_used: if given, the floats at the start of `part` that earlier flushes of the same call own (their
// launches may still be running on the other stream); this flush takes the next ones
d2ft_status weight_grad_flush(WeightGradBatch* b, const d2ft_block_desc* d, const Dims& s, float* part, size_t part_floats,
                              hipStream_t st, size_t* part_used = nullptr, int max_units = 0) {
    if (b->g.n_groups == 0) return D2FT_OK;
    GemmArgs& g = b->g;
    g.K = (int)s.M;
    g.max_units = max_units;
    if (part_used) {
        part += *part_used;
        part_floats -= *part_used;
        *part_used += gemm_grouped_slots(g) * 65536;
    }
    g.partial = part;
    const int accum = (d->flags & D2FT_FLAG_ACCUM_GRADS) ? 1 : 0;
    hipError_t e = hipErrorNotSupported;
    if (gemm_grouped_slots(g) * 65536 <= part_floats) {
        timing_begin(st, "gemm");
        g_timing.label = "gemm_mfma_kernel<256, 256, 64, 2, 4, true, true, 0, false, true, false, 0>";
        for (int i = 0; i < g.n_groups; ++i) g_timing.flops += 2.0 * g.grp[i].M * g.grp[i].N * s.M;
        e = launch_gemm_grouped(&g, st);
        timing_end(st);
    }
    if (e == hipSuccess) {
        // every (workgroup, tile) partial is read once, every output element written once
        const double nbytes = 4.0 * 65536 * g.total_tiles * g.splits;
        D2FT_TRY_BYTES(nbytes, launch_reduce_grouped(s.dtype, g, b->r, accum, st));
    } else if (e == hipErrorNotSupported) {   // an operand the grouped kernel does not take: one launch per gradient
        for (int i = 0; i < g.n_groups; ++i) {
            const GemmGroup& G = g.grp[i];
            const ReduceGroup& R = b->r.grp[i];
            d2ft_status rc;
            if (R.remap == RED_REMAP_F32) {   // queued last: nothing overwrites its slices before the consumer runs
                int splits = 1;
                rc = weight_grad(d, s, G.A, G.lda, G.B, G.ldb, G.M, G.N, part, nullptr, 0, RED_REMAP_NONE, b->r.tbl[0], st,
                                 &splits, false);
                b->f32_splits = splits;
            } else {
                rc = weight_grad(d, s, G.A, G.lda, G.B, G.ldb, G.M, G.N, part, R.out, R.ldo, R.remap, b->r.tbl[R.table], st);
            }
            if (rc != D2FT_OK) return rc;
        }
    } else {
        return D2FT_EDEVICE;
    }
    g.n_groups = 0;
    return D2FT_OK;
}

// bias gradient, first half: column sums of X over row chunks into its own partial region; the reduction
// over the chunks is queued and done for all of a block's biases by one launch (flush_bias_grads)
d2ft_status bias_grad(const Dims& s, const void* X, long ldx, int cols, float* region, void* out, int remap_cols,
                      ColReduceBatch* batch, hipStream_t st) {
    const int chunks = pick_chunks(s.M);
    D2FT_TRY_BYTES(1.0 * s.M * cols * s.es, launch_colsum(s.dtype, X, ldx, (int)s.M, cols, region, chunks, st));
    ColReduceJob& j = batch->job[batch->n++];
    j.partial = region;
    j.out = out;
    j.chunks = chunks;
    j.cols = cols;
    j.remap_cols = remap_cols;
    return D2FT_OK;
}

// bias gradient whose first half a producing kernel has already done: `bands` rows of column sums in region
void queue_bias_reduce(ColReduceBatch* batch, const float* region, int bands, int cols, void* out, int remap_cols) {
    ColReduceJob& j = batch->job[batch->n++];
    j.partial = region;
    j.out = out;
    j.chunks = bands;
    j.cols = cols;
    j.remap_cols = remap_cols;
}

d2ft_status flush_bias_grads(const d2ft_block_desc* d, const Dims& s, ColReduceBatch* batch, const Remap64& tbl_a,
                             const Remap64& tbl_b, hipStream_t st) {
    double nbytes = 0;
    for (int i = 0; i < batch->n; ++i) nbytes += 4.0 * batch->job[i].chunks * batch->job[i].cols;
    D2FT_TRY_BYTES(nbytes, launch_col_reduce_batch(s.dtype, *batch, tbl_a, tbl_b, (d->flags & D2FT_FLAG_ACCUM_GRADS) ? 1 : 0, st));
    batch->n = 0;
    return D2FT_OK;
}

}  // namespace

void launch_signal_next(hipEvent_t ev) { g_launch_signal = ev; }
bool launch_signal_pending() { return g_launch_signal != nullptr; }
hipEvent_t launch_signal_take() {
    hipEvent_t ev = g_launch_signal;
    g_launch_signal = nullptr;
    return ev;
}
}  // namespace d2ft

using namespace d2ft;

extern "C" {

d2ft_status d2ft_timing_enable(int32_t on) {
    // finished records go back to the event pool
    for (TimingRec& r : g_timing.recs) {
        g_timing.pool.push_back(r.a);
        g_timing.pool.push_back(r.b);
    }
    g_timing.recs.clear();
    g_timing.on = on != 0;
    g_timing.open = false;
    return D2FT_OK;
}

int32_t d2ft_timing_read(d2ft_kernel_time* out, int32_t max_entries) {
    if (!out || max_entries < 0) return -1;
    std::map<std::string, d2ft_kernel_time> agg;
    for (TimingRec& r : g_timing.recs) {
        if (hipEventSynchronize(r.b) != hipSuccess) return -1;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return -1;
        d2ft_kernel_time& k = agg[r.label];
        if (k.launches == 0) {
            memset(&k, 0, sizeof(k));
            strncpy(k.name, r.label.c_str(), sizeof(k.name) - 1);
        }
        k.launches += 1;
        k.ms += ms;
        k.flops += r.flops;
        k.bytes += r.bytes;
    }
    int32_t n = 0;
    for (auto& kv : agg) {
        if (n >= max_entries) break;
        out[n++] = kv.second;
    }
    return n;
}

d2ft_status d2ft_join(void* hip_stream) { return join_pending(static_cast<hipStream_t>(hip_stream)); }

const char* d2ft_status_string(d2ft_status status) {
    switch (status) {
        case D2FT_OK: return "ok";
        case D2FT_EINVAL: return "invalid argument (null or misaligned pointer, bad enum, op code or score)";
        case D2FT_ESHAPE: return "unsupported shape or workspace too small";
        case D2FT_EDEVICE: return "HIP error";
    }
    return "unknown status";
}

size_t d2ft_block_saved_bytes(const d2ft_block_desc* desc) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return 0;
    return saved_layout(dims_of(desc)).total;
}

size_t d2ft_block_scratch_bytes(const d2ft_block_desc* desc) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return 0;
    return scratch_layout(dims_of(desc)).total;
}

d2ft_status d2ft_compact_heads(const uint8_t* ops, int32_t heads, int32_t* live, int32_t* n_full, int32_t* n_live) {
    return compact(ops, heads, live, n_full, n_live);
}

static bool grads_aligned(const d2ft_block_grads* grads) {
    const void* gp[] = {grads->ln1_g, grads->ln1_b, grads->w_qkv, grads->b_qkv, grads->w_o, grads->b_o,
                        grads->ln2_g, grads->ln2_b, grads->w1, grads->b1, grads->w2, grads->b2,
                        grads->lora_a_q, grads->lora_a_v, grads->lora_b_q, grads->lora_b_v};
    for (const void* p : gp)
        if (p && !aligned16(p)) return false;
    return true;
}

// Which half of a block a call works on.  The public block calls run both; the micro-batched calls run
// the attention half per micro-batch (its op codes differ) and, when the feed-forward network is not
// gated, the feed-forward half once for the whole batch.
enum { PART_BOTH = 0, PART_ATTN = 1, PART_MLP = 2 };

// Forward of a block or of one half of it.  Arguments are validated by the callers.
//   PART_ATTN: y receives x1 = x + attention residual;   PART_MLP: x is x1.
//   sva / svm: where the attention-side / feed-forward-side fields of SavedLayout live (both are the
//   start of the one saved buffer for PART_BOTH)
//   mask: NULL, or the micro-batches' own codes when ops is their union (see micro_union below)
static d2ft_status block_fwd_impl(const d2ft_block_desc* desc, const d2ft_block_weights* w, const uint8_t* ops,
                                  const void* x, void* y, char* sva, char* svm, void* scratch, hipStream_t st, int part,
                                  const MicroMask* mask = nullptr) {
    int32_t live[D2FT_MAX_HEADS], nf = 0, nl = 0;
    d2ft_status cs = compact(ops, desc->heads, live, &nf, &nl);
    if (cs != D2FT_OK) return cs;
    cs = join_pending(st);   // an earlier backward call may still read the buffers this call writes
    if (cs != D2FT_OK) return cs;

    const Dims s = dims_of(desc);
    const SavedLayout SL = saved_layout(s);
    const ScratchLayout WL = scratch_layout(s);
    char* ws = static_cast<char*>(scratch);
    const int M = (int)s.M;
    const bool gate = (desc->flags & D2FT_FLAG_GATE_FFN) != 0;
    if (part != PART_BOTH && gate) return D2FT_EINVAL;   // a gated feed-forward slice goes with its head
    char* sv = sva;

    const void* x1 = x;   // all heads shortcut: the attention residual is x itself
    if (part != PART_MLP && nl > 0) {
        void* u = sv + SL.u;
        D2FT_TRY_BYTES(2.0 * s.M * s.D * s.es + 8.0 * s.M, launch_ln_fwd(s.dtype, x, w->ln1_g, w->ln1_b, u, (float*)(sv + SL.mean1), (float*)(sv + SL.rstd1), M,
                               s.D, desc->ln_eps, st));
        // Q, K, V of the live heads only
        GemmArgs g = gemm_base();
        fill_qkv_table(g.tbl, live, nl, s.H);
        g.A = u; g.a_rs = s.D; g.a_cs = 1;
        g.M = M; g.N = nl * 192; g.K = s.D;
        g.C = sv + SL.qkv; g.ldc = nl * 192;
        g.bias = w->b_qkv; g.bias_remap = 1;
        if (s.r > 0) {
            HeadList hl; hl.n = nl;
            for (int j = 0; j < nl; ++j) hl.h[j] = (uint8_t)live[j];
            D2FT_TRY(launch_lora_merge(s.dtype, w->w_qkv, w->lora_a_q, w->lora_a_v, w->lora_b_q, w->lora_b_v,
                                       sv + SL.weff, hl, nl, s.H, s.D, s.r, desc->lora_scale, st));
            g.B = sv + SL.weff; g.b_rs = 1; g.b_cs = s.D; g.remap = REMAP_NONE;
        } else {
            g.B = w->w_qkv; g.b_rs = 1; g.b_cs = s.D; g.remap = REMAP_B_N;
        }
        D2FT_TRY_UNTIMED(run_gemm(g, desc, st));
        // softmax attention per (image, live head); log-sum-exp kept for p_f heads only
        D2FT_TRY(run_attn_fwd(desc, sv + SL.qkv, nl * 192, sv + SL.o, nl * 64, (float*)(sv + SL.lse), s.B, s.T, nl, nf,
                              st, mask));
        // x1 = x + O Wo_live^T + b_o
        GemmArgs p = gemm_base();
        fill_head_table(p.tbl, live, nl);
        p.A = sv + SL.o; p.a_rs = nl * 64; p.a_cs = 1;
        p.B = w->w_o; p.b_rs = 1; p.b_cs = (long)s.H * 64; p.remap = REMAP_B_K;
        p.M = M; p.N = s.D; p.K = nl * 64;
        p.C = (part == PART_ATTN) ? y : (void*)(sv + SL.x1); p.ldc = s.D;
        p.bias = w->b_o;
        p.residual = x; p.ldr = s.D;
        // micro-batches with their own codes: the O block of a skipped pair is zero, so a tile need not walk it
        hipError_t ek = mask ? run_gemm_kseg(p, desc, *mask, mask->live, s.T, 64, st) : hipErrorNotSupported;
        if (ek == hipErrorNotSupported) D2FT_TRY_UNTIMED(run_gemm(p, desc, st));
        else if (ek != hipSuccess) return D2FT_EDEVICE;
        x1 = p.C;
        // the backward multiplies the saved O of the p_f positions over the whole batch: a pair that
        // was forward-only in its micro-batch must not reach the gradient of W_o
        if (mask) D2FT_TRY(launch_zero_pairs(s.dtype, sv + SL.o, nullptr, nl * 64, s.B, s.T, nf, 64, PAIRS_FORWARD_ONLY, *mask, st));
    }
    if (part == PART_ATTN) {
        if (nl == 0) {   // x1 is x: the caller wants it in y
            timing_begin(st, "copy");
            const hipError_t e = hipMemcpyAsync(y, x, (size_t)s.M * s.D * s.es, hipMemcpyDeviceToDevice, st);
            timing_end(st);
            if (e != hipSuccess) return D2FT_EDEVICE;
        }
        return D2FT_OK;
    }
    sv = svm;
    if (gate && nl == 0) {   // no live subnet: the block is the identity (neither bias is applied)
        timing_begin(st, "copy");
        const hipError_t e = hipMemcpyAsync(y, x, (size_t)s.M * s.D * s.es, hipMemcpyDeviceToDevice, st);
        timing_end(st);
        return e == hipSuccess ? D2FT_OK : D2FT_EDEVICE;
    }
    // feed-forward columns in use: all of them, or the slices of the live heads in compacted order
    const int slice = gate ? s.Dm / s.H : 0;
    const int n_hid = gate ? nl * slice : s.Dm;
    Remap64 ffn_tbl;
    memset(&ffn_tbl, 0, sizeof(ffn_tbl));
    if (gate) fill_ffn_table(ffn_tbl, live, nl, slice);
    void* v = sv + SL.v;
    D2FT_TRY_BYTES(2.0 * s.M * s.D * s.es + 8.0 * s.M, launch_ln_fwd(s.dtype, x1, w->ln2_g, w->ln2_b, v, (float*)(sv + SL.mean2), (float*)(sv + SL.rstd2), M, s.D,
                           desc->ln_eps, st));
    {   // z = v W1^T + b1, g = GELU(z)
        GemmArgs g = gemm_base();
        g.tbl = ffn_tbl;
        g.A = v; g.a_rs = s.D; g.a_cs = 1;
        g.B = w->w1; g.b_rs = 1; g.b_cs = s.D; g.remap = gate ? REMAP_B_N : REMAP_NONE;
        g.M = M; g.N = n_hid; g.K = s.D;
        g.C = sv + SL.g; g.ldc = n_hid;
        g.bias = w->b1; g.bias_remap = gate ? 1 : 0;
        g.act = ACT_GELU; g.Z = sv + SL.z; g.ldz = n_hid;
        // a subnet skipped in a micro-batch adds nothing to that micro-batch's rows: left out of the product, or
        // zeroed behind it
        hipError_t es = (gate && mask) ? run_gemm_segments(g, desc, *mask, mask->live, s.T, slice, st) : hipErrorNotSupported;
        if (es == hipErrorNotSupported) {
            D2FT_TRY_UNTIMED(run_gemm(g, desc, st));
            if (gate && mask) D2FT_TRY(launch_zero_pairs(s.dtype, sv + SL.g, sv + SL.z, n_hid, s.B, s.T, nl, slice, PAIRS_SKIPPED, *mask, st));
        } else if (es != hipSuccess) {
            return D2FT_EDEVICE;
        }
    }
    {   // y = x1 + g W2^T + b2
        GemmArgs g = gemm_base();
        g.tbl = ffn_tbl;
        g.A = sv + SL.g; g.a_rs = n_hid; g.a_cs = 1;
        g.B = w->w2; g.b_rs = 1; g.b_cs = s.Dm; g.remap = gate ? REMAP_B_K : REMAP_NONE;
        g.M = M; g.N = s.D; g.K = n_hid;
        g.C = y; g.ldc = s.D;
        g.bias = w->b2;
        g.residual = x1; g.ldr = s.D;
        // micro-batches with their own codes: g is zero where a slice was skipped, so a tile need not walk it
        hipError_t ek = (gate && mask) ? run_gemm_kseg(g, desc, *mask, mask->live, s.T, slice, st) : hipErrorNotSupported;
        if (ek == hipErrorNotSupported) D2FT_TRY_UNTIMED(run_gemm(g, desc, st));
        else if (ek != hipSuccess) return D2FT_EDEVICE;
        // the backward multiplies the saved g and GELU' of the p_f slices over the whole batch: zero what
        // was forward-only in its micro-batch (dz = (dy W2) * GELU' is then zero there too)
        if (gate && mask) D2FT_TRY(launch_zero_pairs(s.dtype, sv + SL.g, sv + SL.z, n_hid, s.B, s.T, nf, slice, PAIRS_FORWARD_ONLY, *mask, st));
    }
    return D2FT_OK;
}

d2ft_status d2ft_block_fwd(const d2ft_block_desc* desc, const d2ft_block_weights* w, const uint8_t* ops,
                           const void* x, void* y, void* saved, void* scratch, void* hip_stream) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!weights_ok(desc, w) || !ops || !x || !y || !saved || !scratch || x == y) return D2FT_EINVAL;
    if (!aligned16(x) || !aligned16(y) || ((uintptr_t)saved & 255) || ((uintptr_t)scratch & 255)) return D2FT_EINVAL;
    return block_fwd_impl(desc, w, ops, x, y, static_cast<char*>(saved), static_cast<char*>(saved), scratch,
                          static_cast<hipStream_t>(hip_stream), PART_BOTH);
}

// Backward of a block or of one half of it.  Arguments are validated by the callers.
//   PART_MLP:  x is x1, dy the gradient of the block output, dx receives dx1 (the gradient of x1)
//   PART_ATTN: dy is dx1 and may be the same buffer as dx (rows are rewritten in place)
static d2ft_status block_bwd_impl(const d2ft_block_desc* desc, const d2ft_block_weights* w, const uint8_t* ops,
                                  const void* x, const void* dy, void* dx, const d2ft_block_grads* grads,
                                  const char* sva, const char* svm, void* scratch, hipStream_t st, int half,
                                  const MicroMask* mask = nullptr) {
    int32_t live[D2FT_MAX_HEADS], nf = 0, nl = 0;
    d2ft_status cs = compact(ops, desc->heads, live, &nf, &nl);
    if (cs != D2FT_OK) return cs;

    const Dims s = dims_of(desc);
    const SavedLayout SL = saved_layout(s);
    const ScratchLayout WL = scratch_layout(s);
    const char* sv = svm;
    char* ws = static_cast<char*>(scratch);
    const int M = (int)s.M;
    const int accum = (desc->flags & D2FT_FLAG_ACCUM_GRADS) ? 1 : 0;
    float* part = (float*)(ws + WL.part);
    float* colpart = (float*)(ws + WL.colpart);
    float* ln_part = colpart + 4 * WL.colpart_stride;
    ColReduceBatch bias_batch;
    memset(&bias_batch, 0, sizeof(bias_batch));
    WeightGradBatch wgrads;
    weight_grad_batch_init(&wgrads, desc);
    Remap64 none;
    memset(&none, 0, sizeof(none));
    const void* x1 = (half != PART_MLP && nl > 0) ? (const void*)(sva + SL.x1) : x;
    d2ft_status rc;
    // LoRA: dW_eff of the p_f heads rides in the weight-gradient batch as an fp32 product; the adapters' gradients
    // are projected from it once the batch has run
    bool lora_queued = false;
    HeadList lora_heads; lora_heads.n = 0;
    // Side stream (see SideStream): for the whole-block matrix-core path, unless the caller asks for one stream,
    // per-kernel timing is on (its durations are those of kernels running alone) or the stream is being captured.
    SideStream* side = nullptr;
    if (half == PART_BOTH && wgrads.enabled && !(desc->flags & D2FT_FLAG_ONE_STREAM) && !g_timing.on) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cap) == hipSuccess && cap == hipStreamCaptureStatusNone) side = side_stream();
    }
    bool side_used = false;   // a join is due at the call's end
    // An earlier call that deferred its join.  If this call has the same shape (hence the same scratch layout)
    // and defers too, what may still be running of that call are its weight-gradient launches: they read its dz
    // and its fused column sums, of which consecutive calls use alternating copies, and dx1 and dQKV.  This call
    // then waits only before it writes dx1 (join_late), by when they have long ended - and since that wait
    // covers the whole earlier call, the copies this call writes now were last read two calls ago, behind the
    // wait of the call before.  Otherwise it waits for everything now.
    bool join_late = false;
    if (SideStream* P = side_stream(false); P && P->pending) {
        const Dims& q = P->pending_dims;
        const bool same = q.B == s.B && q.T == s.T && q.D == s.D && q.H == s.H && q.Dm == s.Dm && q.r == s.r && q.dtype == s.dtype;
        if (side && same && (desc->flags & D2FT_FLAG_DEFER_JOIN)) {
            P->pending = false;
            join_late = true;
        } else {
            const d2ft_status rj = join_pending(st);
            if (rj != D2FT_OK) return rj;
        }
    }
    auto late_join = [&]() -> d2ft_status {   // before the first write to what the earlier call's last launch reads
        if (!join_late) return D2FT_OK;
        join_late = false;
        return hipStreamWaitEvent(st, side->join, 0) == hipSuccess ? D2FT_OK : D2FT_EDEVICE;
    };
    // the set of fused column-sum regions of this call
    const int parity = side ? (side->parity ^= 1) : 0;
    const size_t cf = parity * WL.colfuse_set;
    char* const dz_buf = ws + WL.dz + parity * WL.dz_alt;   // dz of this call
    // Where the join is deferred the bias reductions go to the side stream with the last weight gradients (the
    // caller's stream then ends the call with LayerNorm 1's backward); where the call ends joined they stay on
    // the caller's stream, which would otherwise wait for them.
    const bool bias_on_side = side && (desc->flags & D2FT_FLAG_DEFER_JOIN);
    hipStream_t const st_main = st;
    hipStream_t const st_side = side ? side->stream : st;
    size_t part_used = 0;   // floats of `part` owned by weight-gradient launches that may still be running
    // the weight gradients collected so far (and what follows from them) on stream `st`
    auto flush_wgrads = [&](hipStream_t st, int max_units = 0) -> d2ft_status {
        float* const mine = part + part_used;
        const d2ft_status rw = weight_grad_flush(&wgrads, desc, s, part, WL.part_floats, st, &part_used, max_units);
        if (rw != D2FT_OK) return rw;
        if (lora_queued) {
            lora_queued = false;
            const long elems = (long)lora_heads.n * 192 * s.D;
            const float* G = wgrads.f32_splits > 0 ? mine : (const float*)(ws + WL.lora_g);
            D2FT_TRY(launch_lora_project(s.dtype, G, wgrads.f32_splits > 0 ? wgrads.f32_splits : 1, elems, w->lora_a_q,
                                         w->lora_a_v, w->lora_b_q, w->lora_b_v, grads->lora_a_q, grads->lora_a_v,
                                         grads->lora_b_q, grads->lora_b_v, lora_heads, s.H, s.D, s.r, desc->lora_scale, accum, st));
        }
        return D2FT_OK;
    };
    // hand the weight gradients collected so far to the side stream, which picks them up behind what the
    // caller's stream holds now; without a side stream nothing happens here and they wait for the call's end
    // Zero fills of the gradient slices of subnets that are not p_f: nothing in the call reads them and the
    // reductions write other slices, so with the join deferred they wait for the next hand-over and ride on the
    // side stream behind it instead of taking a turn on the caller's.
    HeadList zero_list; zero_list.n = 0;
    bool zero_heads_due = false, zero_ffn_due = false;
    int zero_slice = 0;
    auto launch_zeros = [&](hipStream_t st) -> d2ft_status {
        if (zero_ffn_due) {
            zero_ffn_due = false;
            D2FT_TRY(launch_zero_ffn_slices(s.dtype, zero_list, zero_slice, s.D, s.Dm, grads->w1, grads->b1, grads->w2, st));
        }
        if (zero_heads_due) {
            zero_heads_due = false;
            D2FT_TRY(launch_zero_head_slices(s.dtype, zero_list, s.H, s.D, s.r, grads->w_qkv, grads->b_qkv, grads->w_o,
                                             grads->lora_a_q, grads->lora_a_v, grads->lora_b_q, grads->lora_b_v, st));
        }
        return D2FT_OK;
    };
    bool fork_recorded = false;   // the last launch on the caller's stream completes side->fork itself
    auto hand_over = [&](int max_units) -> d2ft_status {
        if (!side || wgrads.g.n_groups == 0) return D2FT_OK;
        if (fork_recorded) {
            fork_recorded = false;
            if (hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess) return D2FT_EDEVICE;
        } else if (!side_fork(side, st_main)) {
            return D2FT_EDEVICE;
        }
        side_used = true;
        const d2ft_status rw = flush_wgrads(st_side, max_units);
        return rw != D2FT_OK ? rw : launch_zeros(st_side);
    };
    // the call's last launches: the collected weight gradients, then the bias reductions, then the join
    auto finish = [&](const Remap64& tbl_a, const Remap64& tbl_b) -> d2ft_status {
        const d2ft_status rw = flush_wgrads(st_main);
        if (rw != D2FT_OK) return rw;
        const d2ft_status rz = launch_zeros(st_main);   // no hand-over took them along
        if (rz != D2FT_OK) return rz;
        if (bias_batch.n > 0) {
            const d2ft_status rb = flush_bias_grads(desc, s, &bias_batch, tbl_a, tbl_b, st_main);
            if (rb != D2FT_OK) return rb;
        }
        const d2ft_status rl = late_join();
        if (rl != D2FT_OK) return rl;
        if (side_used) {
            if (hipEventRecord(side->join, st_side) != hipSuccess) return D2FT_EDEVICE;
            if (desc->flags & D2FT_FLAG_DEFER_JOIN) {   // the next call on this device, or d2ft_join, waits for it
                side->pending = true;
                side->pending_dims = s;
            } else if (hipStreamWaitEvent(st_main, side->join, 0) != hipSuccess) {
                return D2FT_EDEVICE;
            }
        }
        return D2FT_OK;
    };

    // ---- feed-forward network: all of it, or (gated) the slices of the p_f heads, a prefix of the compacted layout ----
    const bool gate = (desc->flags & D2FT_FLAG_GATE_FFN) != 0;
    if (half != PART_BOTH && gate) return D2FT_EINVAL;   // a gated feed-forward slice goes with its head
    const int slice = gate ? s.Dm / s.H : 0;
    const int ld_hid = gate ? nl * slice : s.Dm;      // row stride of the saved z and g
    const int n_hid = gate ? nf * slice : s.Dm;       // hidden units that take part in backward
    Remap64 ffn_tbl;
    memset(&ffn_tbl, 0, sizeof(ffn_tbl));
    if (gate) fill_ffn_table(ffn_tbl, live, nf, slice);
    if (gate && !accum) {   // feed-forward slices of subnets that are not p_f: +0.0
        HeadList nonfull; nonfull.n = 0;
        for (int h = 0; h < s.H; ++h)
            if (ops[h] != D2FT_OP_FULL) nonfull.h[nonfull.n++] = (uint8_t)h;
        if (bias_on_side) {
            zero_list = nonfull;
            zero_slice = slice;
            zero_ffn_due = true;
        } else {
            D2FT_TRY(launch_zero_ffn_slices(s.dtype, nonfull, slice, s.D, s.Dm, grads->w1, grads->b1, grads->w2, st));
        }
        if (nl == 0 && grads->b2 && w->b2)   // bias was not applied: its gradient is zero
            D2FT_TRY(launch_reduce_partials(s.dtype, colpart, 0, 0, 1, s.D, grads->b2, s.D, RED_REMAP_NONE, none, 0, st));
        if (nf == 0) {
            if (grads->ln2_g) D2FT_TRY(launch_reduce_partials(s.dtype, colpart, 0, 0, 1, s.D, grads->ln2_g, s.D, RED_REMAP_NONE, none, 0, st));
            if (grads->ln2_b) D2FT_TRY(launch_reduce_partials(s.dtype, colpart, 0, 0, 1, s.D, grads->ln2_b, s.D, RED_REMAP_NONE, none, 0, st));
        }
    }
    // The LayerNorm backward of the feed-forward half reads dy and writes dx1: where it runs it also sums
    // their columns, which are the gradients of b2 and b_o; otherwise those are column-sum passes of their own.
    const bool ln2_runs = half != PART_ATTN && n_hid > 0;
    const bool ln2_sums = ln2_runs && ln_bwd_sums_supported(s.D);
    const bool want_b2 = half != PART_ATTN && grads->b2 && w->b2 && (!gate || nl > 0);
    const bool want_bo = half != PART_MLP && grads->b_o && w->b_o && nl > 0;
    if (want_b2 && !ln2_sums) {
        rc = bias_grad(s, dy, s.D, s.D, colpart + 0 * WL.colpart_stride, grads->b2, 0, &bias_batch, st);
        if (rc != D2FT_OK) return rc;
    }
    // gradient of x1.  It is dy when the feed-forward half is not run here: handed over by the caller
    // (PART_ATTN), or gated with no p_f subnet (the residual route alone).
    const void* dx1 = dy;
    int b1_bands = 0;
    if (half != PART_ATTN && n_hid > 0) {
        if (grads->w2) {   // dW2[:, hidden] = dy^T g
            rc = weight_grad_queue(&wgrads, desc, s, dy, s.D, sv + SL.g, ld_hid, s.D, n_hid, part, grads->w2, s.Dm,
                                   gate ? RED_REMAP_COLS : RED_REMAP_NONE, ffn_tbl, 0, st);
            if (rc != D2FT_OK) return rc;
        }
        {   // dz = (dy W2[:, hidden]) * GELU'(z)
            GemmArgs g = gemm_base();
            g.tbl = ffn_tbl;
            g.A = dy; g.a_rs = s.D; g.a_cs = 1;
            g.B = w->w2; g.b_rs = s.Dm; g.b_cs = 1;   // B(k = width index, n = hidden index) = W2[k][n]
            g.remap = gate ? REMAP_B_N : REMAP_NONE;
            g.M = M; g.N = n_hid; g.K = s.D;
            g.C = dz_buf; g.ldc = n_hid;
            g.act = ACT_DGELU; g.Z = const_cast<char*>(sv + SL.z); g.ldz = ld_hid;
            if (grads->b1 && on_mfma_path(g, desc)) g.colsum = (float*)(ws + WL.colfuse_b1 + cf);   // db1 = column sums of dz
            // micro-batches with their own codes: the saved GELU' is zero where a slice was not p_f, so those
            // products need not be formed
            // if the feed-forward weight gradients go to the side stream behind dz, the dz launch itself completes
            // the event that stream waits for
            long ffn_tiles = 0;
            if (grads->w2) ffn_tiles += (long)((s.D + 255) / 256) * ((n_hid + 255) / 256);
            if (grads->w1) ffn_tiles += (long)((n_hid + 255) / 256) * ((s.D + 255) / 256);
            hipEvent_t dz_done = (side && ffn_tiles >= 24) ? side->fork : nullptr;
            hipError_t es = (gate && mask) ? run_gemm_segments(g, desc, *mask, mask->full, s.T, slice, st, &b1_bands, dz_done) : hipErrorNotSupported;
            if (es == hipErrorNotSupported) D2FT_TRY_UNTIMED(run_gemm(g, desc, st, &b1_bands, dz_done));
            else if (es != hipSuccess) return D2FT_EDEVICE;
            if (dz_done && launch_signal_pending()) launch_signal_next(nullptr);   // no launch took it: record it below
            else if (dz_done) fork_recorded = true;
            if (!g.colsum) b1_bands = 0;
        }
        if (grads->w1) {   // dW1[hidden] = dz^T v
            rc = weight_grad_queue(&wgrads, desc, s, dz_buf, n_hid, sv + SL.v, s.D, n_hid, s.D, part, grads->w1, s.D,
                                   gate ? RED_REMAP_ROWS : RED_REMAP_NONE, ffn_tbl, 0, st);
            if (rc != D2FT_OK) return rc;
        }
        // dW2 and dW1 have their operands (dy, g, dz, v: nothing later in the call writes them).  From 24 tiles on
        // they go to the side stream now.  They have a long stretch of the caller's stream beside them and should
        // leave that stream CUs: the launch is held to 128 workgroups, or to two runs of K per tile if that is
        // more.  Measured per step: vit_b16 (72 tiles) 2 runs 8.41 ms, the 3 runs the launch would pick alone 8.56,
        // 1 run 9.10; gated at 7 p_f subnets (42 tiles) 3 runs 7.18 ms, the 6 runs it would pick alone 7.39, 2 runs
        // 7.26, everything in one launch behind the attention backward 7.30.
        if (side) {
            long tiles = 0;
            for (int i = 0; i < wgrads.g.n_groups; ++i)
                tiles += (long)((wgrads.g.grp[i].M + 255) / 256) * ((wgrads.g.grp[i].N + 255) / 256);
            if (tiles >= 24) {
                rc = hand_over((int)(2 * tiles > 128 ? 2 * tiles : 128));
                if (rc != D2FT_OK) return rc;
            }
        }
        fork_recorded = false;   // it stood for this point of the stream only
        if (grads->b1 && b1_bands > 0) {
            queue_bias_reduce(&bias_batch, (const float*)(ws + WL.colfuse_b1 + cf), b1_bands, n_hid, grads->b1, gate ? 2 : 0);
        } else if (grads->b1) {
            rc = bias_grad(s, dz_buf, n_hid, n_hid, colpart + 1 * WL.colpart_stride, grads->b1, gate ? 2 : 0,
                           &bias_batch, st);
            if (rc != D2FT_OK) return rc;
        }
        {   // dv = dz W1[hidden]
            GemmArgs g = gemm_base();
            g.tbl = ffn_tbl;
            g.A = dz_buf; g.a_rs = n_hid; g.a_cs = 1;
            g.B = w->w1; g.b_rs = s.D; g.b_cs = 1; g.remap = gate ? REMAP_B_K : REMAP_NONE;
            g.M = M; g.N = s.D; g.K = n_hid;
            g.C = ws + WL.dv; g.ldc = s.D;
            // micro-batches with their own codes: dz is zero where a slice was not p_f
            hipError_t ek = (gate && mask) ? run_gemm_kseg(g, desc, *mask, mask->full, s.T, slice, st) : hipErrorNotSupported;
            if (ek == hipErrorNotSupported) D2FT_TRY_UNTIMED(run_gemm(g, desc, st));
            else if (ek != hipSuccess) return D2FT_EDEVICE;
        }
        if (grads->ln2_g || grads->ln2_b) {
            const int chunks = pick_chunks(s.M);
            float* pg = ln_part;
            float* pb = ln_part + WL.colpart_stride;
            D2FT_TRY(launch_ln_param_grad(s.dtype, ws + WL.dv, x1, (const float*)(sv + SL.mean2),
                                          (const float*)(sv + SL.rstd2), pg, pb, M, s.D, chunks, st));
            if (grads->ln2_g)
                D2FT_TRY(launch_reduce_partials(s.dtype, pg, chunks, s.D, 1, s.D, grads->ln2_g, s.D, RED_REMAP_NONE, none, accum, st));
            if (grads->ln2_b)
                D2FT_TRY(launch_reduce_partials(s.dtype, pb, chunks, s.D, 1, s.D, grads->ln2_b, s.D, RED_REMAP_NONE, none, accum, st));
        }
        // dx1 = dy + LN2bwd(dv); with no p_f head this already is dx (residual route only)
        void* out = (half == PART_BOTH && nf > 0) ? (void*)(ws + WL.dx1) : dx;
        rc = late_join();
        if (rc != D2FT_OK) return rc;
        if (ln2_sums && (want_b2 || want_bo)) {
            float* sum_res = want_b2 ? (float*)(ws + WL.colfuse_b2 + cf) : nullptr;
            float* sum_out = want_bo ? (float*)(ws + WL.colfuse_bo + cf) : nullptr;
            D2FT_TRY_BYTES(4.0 * s.M * s.D * s.es + 8.0 * s.M, launch_ln_bwd_sums(s.dtype, ws + WL.dv, x1, (const float*)(sv + SL.mean2),
                                        (const float*)(sv + SL.rstd2), w->ln2_g, dy, out, M, s.D, sum_res, sum_out, st));
            const int bands = ln_bwd_sums_bands(M);
            if (want_b2) queue_bias_reduce(&bias_batch, sum_res, bands, s.D, grads->b2, 0);
            if (want_bo) queue_bias_reduce(&bias_batch, sum_out, bands, s.D, grads->b_o, 0);
        } else {
            D2FT_TRY_BYTES(4.0 * s.M * s.D * s.es + 8.0 * s.M, launch_ln_bwd(s.dtype, ws + WL.dv, x1, (const float*)(sv + SL.mean2), (const float*)(sv + SL.rstd2),
                                   w->ln2_g, dy, out, M, s.D, st));
        }
        dx1 = out;
    }
    if (half == PART_MLP) return finish(none, ffn_tbl);

    // ---- attention side ----
    sv = sva;
    rc = late_join();   // if the feed-forward half did not run
    if (rc != D2FT_OK) return rc;
    if (want_bo && !ln2_sums) {
        rc = bias_grad(s, dx1, s.D, s.D, colpart + 2 * WL.colpart_stride, grads->b_o, 0, &bias_batch, st);
        if (rc != D2FT_OK) return rc;
    }
    // heads that are not p_f: gradient slices are +0.0 in overwrite mode, untouched in accumulate mode
    if (!accum) {
        HeadList nonfull; nonfull.n = 0;
        for (int h = 0; h < s.H; ++h)
            if (ops[h] != D2FT_OP_FULL) nonfull.h[nonfull.n++] = (uint8_t)h;
        if (bias_on_side) {
            zero_list = nonfull;
            zero_heads_due = true;
        } else {
            D2FT_TRY(launch_zero_head_slices(s.dtype, nonfull, s.H, s.D, s.r, grads->w_qkv, grads->b_qkv, grads->w_o,
                                             grads->lora_a_q, grads->lora_a_v, grads->lora_b_q, grads->lora_b_v, st));
        }
        if (nl == 0 && grads->b_o && w->b_o) {   // bias was not applied: its gradient is zero
            // a [1][D] "partial" of zero splits writes +0.0
            D2FT_TRY(launch_reduce_partials(s.dtype, colpart, 0, 0, 1, s.D, grads->b_o, s.D, RED_REMAP_NONE, none, 0, st));
        }
        if (nf == 0) {
            if (grads->ln1_g) D2FT_TRY(launch_reduce_partials(s.dtype, colpart, 0, 0, 1, s.D, grads->ln1_g, s.D, RED_REMAP_NONE, none, 0, st));
            if (grads->ln1_b) D2FT_TRY(launch_reduce_partials(s.dtype, colpart, 0, 0, 1, s.D, grads->ln1_b, s.D, RED_REMAP_NONE, none, 0, st));
        }
    }
    if (nf == 0) {
        if (dx1 != dx) {   // the gradient passes by the residual route unchanged
            timing_begin(st, "copy");
            const hipError_t e = hipMemcpyAsync(dx, dx1, (size_t)s.M * s.D * s.es, hipMemcpyDeviceToDevice, st);
            timing_end(st);
            if (e != hipSuccess) return D2FT_EDEVICE;
        }
        return finish(none, ffn_tbl);
    }

    const long ldq = (long)nl * 192, ldo = (long)nl * 64;
    const long ld_do = (long)nf * 64, ld_dq = (long)nf * 192;
    Remap64 head_tbl, qkv_tbl;
    memset(&head_tbl, 0, sizeof(head_tbl));
    memset(&qkv_tbl, 0, sizeof(qkv_tbl));
    fill_head_table(head_tbl, live, nf);
    fill_qkv_table(qkv_tbl, live, nf, s.H);
    {   // dO = dx1 Wo[:, p_f heads]
        GemmArgs g = gemm_base();
        g.tbl = head_tbl;
        g.A = dx1; g.a_rs = s.D; g.a_cs = 1;
        g.B = w->w_o; g.b_rs = (long)s.H * 64; g.b_cs = 1; g.remap = REMAP_B_N;
        g.M = M; g.N = nf * 64; g.K = s.D;
        g.C = ws + WL.d_o; g.ldc = ld_do;
        D2FT_TRY_UNTIMED(run_gemm(g, desc, st));
    }
    if (grads->w_o) {   // dWo[:, head cols] = dx1^T O_h
        rc = weight_grad_queue(&wgrads, desc, s, dx1, s.D, sv + SL.o, ldo, s.D, nf * 64, part, grads->w_o, (long)s.H * 64,
                               RED_REMAP_COLS, head_tbl, 1, st);
        if (rc != D2FT_OK) return rc;
    }
    // the matrix-core attention backward also leaves per-image column sums of dQKV: the QKV bias gradient
    const bool fuse_bqkv = grads->b_qkv && (mask || attn_bwd_on_mfma(desc, s.T, ldq, ldo, ld_do, ld_dq));
    float* bqkv_part = fuse_bqkv ? (float*)(ws + WL.colfuse_bqkv + cf) : nullptr;
    const bool want_lora = s.r > 0 && (grads->lora_a_q || grads->lora_a_v || grads->lora_b_q || grads->lora_b_v);
    // If the side stream takes over right behind the attention backward (nothing else is launched on the caller's
    // stream between the two), that launch itself completes the event the side stream waits for.
    const bool room = wgrads.g.n_groups < kMaxGemmGroups;   // dWqkv (or the LoRA product) joins the batch
    const bool lora_batched = want_lora && !grads->w_qkv && room;
    const bool quiet = room && (fuse_bqkv || !grads->b_qkv) && (!want_lora || lora_batched);
    hipEvent_t attn_done = (side && dx1 != dx && quiet && (!lora_batched || bias_on_side)) ? side->fork : nullptr;
    D2FT_TRY(run_attn_bwd(desc, sv + SL.qkv, ldq, sv + SL.o, ldo, (const float*)(sv + SL.lse), ws + WL.d_o, ld_do,
                          ws + WL.dqkv, ld_dq, (float*)(ws + WL.delta), bqkv_part, s.B, s.T, nf, st, mask, attn_done));
    if (attn_done && launch_signal_pending()) launch_signal_next(nullptr);   // no launch took it: recorded below
    else if (attn_done) fork_recorded = true;
    const void* u = sv + SL.u;
    if (grads->w_qkv && !want_lora) {   // dWqkv = dQKV^T u, rows scattered to the p_f heads' planes
        rc = weight_grad_queue(&wgrads, desc, s, ws + WL.dqkv, ld_dq, u, s.D, nf * 192, s.D, part, grads->w_qkv, s.D,
                               RED_REMAP_ROWS, qkv_tbl, 2, st);
        if (rc != D2FT_OK) return rc;
    } else if (want_lora && !grads->w_qkv && wgrads.enabled && wgrads.g.n_groups < kMaxGemmGroups) {
        // G = dQKV^T u (rows in compacted order) as one more group of the batch, left in fp32
        rc = weight_grad_queue(&wgrads, desc, s, ws + WL.dqkv, ld_dq, u, s.D, nf * 192, s.D, part, ws + WL.lora_g, s.D,
                               RED_REMAP_F32, qkv_tbl, 2, st);
        if (rc != D2FT_OK) return rc;
        lora_queued = true;
        lora_heads.n = nf;
        for (int j = 0; j < nf; ++j) lora_heads.h[j] = (uint8_t)live[j];
    } else if (want_lora) {   // the same product by a launch of its own
        int splits = 1;
        float* const mine = part + part_used;   // behind the partial tiles of launches that may still be running
        rc = weight_grad(desc, s, ws + WL.dqkv, ld_dq, u, s.D, nf * 192, s.D, mine, grads->w_qkv, s.D, RED_REMAP_ROWS, qkv_tbl,
                         st, &splits, grads->w_qkv != nullptr);
        if (rc != D2FT_OK) return rc;
        if (want_lora) {
            HeadList fl; fl.n = nf;
            for (int j = 0; j < nf; ++j) fl.h[j] = (uint8_t)live[j];
            D2FT_TRY(launch_lora_project(s.dtype, mine, splits, (long)nf * 192 * s.D, w->lora_a_q, w->lora_a_v, w->lora_b_q,
                                         w->lora_b_v, grads->lora_a_q, grads->lora_a_v, grads->lora_b_q, grads->lora_b_v,
                                         fl, s.H, s.D, s.r, desc->lora_scale, accum, st));
        }
    }
    if (fuse_bqkv) {
        queue_bias_reduce(&bias_batch, bqkv_part, s.B, nf * 192, grads->b_qkv, 1);   // table a
    } else if (grads->b_qkv) {
        rc = bias_grad(s, ws + WL.dqkv, ld_dq, nf * 192, colpart + 3 * WL.colpart_stride, grads->b_qkv, 1, &bias_batch, st);   // table a
        if (rc != D2FT_OK) return rc;
    }
    // dWo and dWqkv have their operands: they run beside du and the LayerNorm backward (dx1 is only read from
    // here on: with a side stream it is never dx itself).  The bias reductions stay on the caller's stream: with
    // them the two streams end the call at about the same time, and a join that has to wait costs more than
    // the reductions.
    // With LoRA the product is followed by the projection onto the adapters, too long a tail for the side stream
    // beside du alone if the call ends joined (+0.06 ms per step): those then stay on the caller's stream.
    if (dx1 != dx && (!lora_queued || bias_on_side)) {
        const bool forked = side && wgrads.g.n_groups > 0;   // hand_over orders the side stream behind this point
        rc = hand_over(0);   // little is left beside it: as fast as it can
        if (rc != D2FT_OK) return rc;
        if (bias_on_side && forked && bias_batch.n > 0) {
            bool fused_only = true;   // sums a column-sum pass left in the (single) colpart regions stay on the caller's stream
            for (int i = 0; i < bias_batch.n; ++i)
                if (bias_batch.job[i].partial >= colpart && bias_batch.job[i].partial < colpart + 6 * WL.colpart_stride) fused_only = false;
            if (fused_only) {
                rc = flush_bias_grads(desc, s, &bias_batch, qkv_tbl, ffn_tbl, st_side);
                if (rc != D2FT_OK) return rc;
            }
        }
    }
    fork_recorded = false;   // it stood for this point of the stream only
    {   // du = dQKV W_eff (rows of the p_f heads)
        GemmArgs g = gemm_base();
        g.tbl = qkv_tbl;
        g.A = ws + WL.dqkv; g.a_rs = ld_dq; g.a_cs = 1;
        if (s.r > 0) {   // the forward call's merged weights; the p_f heads are their first nf * 192 rows
            g.B = sv + SL.weff; g.remap = REMAP_NONE;
        } else {
            g.B = w->w_qkv; g.remap = REMAP_B_K;
        }
        g.b_rs = s.D; g.b_cs = 1;
        g.M = M; g.N = s.D; g.K = nf * 192;
        g.C = ws + WL.du; g.ldc = s.D;
        // micro-batches with their own codes: the dQKV block of a pair that is not p_f is zero
        hipError_t ek = (mask && s.r == 0) ? run_gemm_kseg(g, desc, *mask, mask->full, s.T, 192, st) : hipErrorNotSupported;
        if (ek == hipErrorNotSupported) D2FT_TRY_UNTIMED(run_gemm(g, desc, st));
        else if (ek != hipSuccess) return D2FT_EDEVICE;
    }
    if (grads->ln1_g || grads->ln1_b) {
        const int chunks = pick_chunks(s.M);
        float* pg = ln_part;
        float* pb = ln_part + WL.colpart_stride;
        D2FT_TRY(launch_ln_param_grad(s.dtype, ws + WL.du, x, (const float*)(sv + SL.mean1),
                                      (const float*)(sv + SL.rstd1), pg, pb, M, s.D, chunks, st));
        if (grads->ln1_g)
            D2FT_TRY(launch_reduce_partials(s.dtype, pg, chunks, s.D, 1, s.D, grads->ln1_g, s.D, RED_REMAP_NONE, none, accum, st));
        if (grads->ln1_b)
            D2FT_TRY(launch_reduce_partials(s.dtype, pb, chunks, s.D, 1, s.D, grads->ln1_b, s.D, RED_REMAP_NONE, none, accum, st));
    }
    if (dx1 == dx) {   // the rows of dx1 are about to be rewritten in place: its weight gradients go first
        rc = flush_wgrads(st_main);
        if (rc != D2FT_OK) return rc;
    }
    // dx = dx1 + LN1bwd(du)
    D2FT_TRY_BYTES(4.0 * s.M * s.D * s.es + 8.0 * s.M, launch_ln_bwd(s.dtype, ws + WL.du, x, (const float*)(sv + SL.mean1), (const float*)(sv + SL.rstd1), w->ln1_g,
                           dx1, dx, M, s.D, st));
    return finish(qkv_tbl, ffn_tbl);
}

d2ft_status d2ft_block_bwd(const d2ft_block_desc* desc, const d2ft_block_weights* w, const uint8_t* ops,
                           const void* x, const void* dy, void* dx, const d2ft_block_grads* grads, const void* saved,
                           void* scratch, void* hip_stream) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!weights_ok(desc, w) || !ops || !x || !dy || !dx || !grads || !saved || !scratch || dy == dx)
        return D2FT_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || ((uintptr_t)saved & 255) || ((uintptr_t)scratch & 255))
        return D2FT_EINVAL;
    if (!grads_aligned(grads)) return D2FT_EINVAL;
    return block_bwd_impl(desc, w, ops, x, dy, dx, grads, static_cast<const char*>(saved), static_cast<const char*>(saved),
                          scratch, static_cast<hipStream_t>(hip_stream), PART_BOTH);
}

// ---- micro-batches: the block calls applied to consecutive image ranges ----
static bool micro_ok(const d2ft_block_desc* desc, int32_t n_micro, const int32_t* mb_images) {
    if (n_micro < 1 || n_micro > D2FT_MAX_MICRO || !mb_images) return false;
    long sum = 0;
    for (int i = 0; i < n_micro; ++i) {
        if (mb_images[i] < 1) return false;
        sum += mb_images[i];
    }
    return sum == desc->batch;
}

// Saved-activation layout of the micro-batched calls.
//   gated feed-forward: one whole SavedLayout per micro-batch (each micro-batch is a block call of its own)
//   otherwise: the attention-side fields per micro-batch, then x1 of the whole batch, then the
//   feed-forward fields of the whole batch (that half does not depend on the op codes, so it runs once)
//   union mode (micro_union below): the plain SavedLayout of the whole batch
struct MicroPlan {
    bool shared_mlp;
    size_t at[D2FT_MAX_MICRO];   // start of micro-batch i's fields
    size_t x1, mlp, total;       // shared_mlp only: whole-batch x1; feed-forward fields begin at mlp
};
static MicroPlan micro_plan(const d2ft_block_desc* desc, int32_t n_micro, const int32_t* mb_images) {
    MicroPlan P;
    memset(&P, 0, sizeof(P));
    P.shared_mlp = (desc->flags & D2FT_FLAG_GATE_FFN) == 0;
    size_t off = 0;
    for (int i = 0; i < n_micro; ++i) {
        d2ft_block_desc d = *desc;
        d.batch = mb_images[i];
        const SavedLayout L = saved_layout(dims_of(&d));
        P.at[i] = off;
        off += P.shared_mlp ? L.x1 : L.total;
    }
    const SavedLayout L = saved_layout(dims_of(desc));
    if (P.shared_mlp) {
        P.x1 = off;
        off += L.mean2 - L.x1;
        P.mlp = off;
        off += L.total - L.mean2;
    }
    P.total = off > L.total ? off : L.total;   // either mode fits
    return P;
}

// Union mode.  With several micro-batches on the matrix-core attention path and every micro-batch
// keeping at least one head live, the block runs ONCE over the whole batch under the union of the
// codes (a head is p_f if it is p_f in any micro-batch, else forward-only if it is live in any):
// the projections then have the whole batch's rows (full tiles, one launch each) instead of a
// fifth of them per launch.  The attention kernels take the micro-batches' own codes as a mask: a
// pair (micro-batch, head) that is skipped gets a zero O block, a pair that is not p_f a zero dQKV
// block and, after the output projection, a zero saved O block, so that every product over the whole
// batch sums exactly the terms the micro-batches' own calls would (plus zeros).  Gated feed-forward
// slices are handled the same way: g and GELU' blocks of skipped pairs are zeroed behind FC1, those of
// forward-only pairs behind FC2.  The price is projection FLOPs on the zero blocks.
static bool micro_union(const d2ft_block_desc* desc, int32_t n_micro, const int32_t* mb_images, const uint8_t* ops,
                        uint8_t* ops_union, MicroMask* mask) {
    if (n_micro < 2 || !attn_on_mfma(desc)) return false;
    const int H = desc->heads;
    for (int h = 0; h < H; ++h) ops_union[h] = D2FT_OP_SKIP;
    for (int i = 0; i < n_micro; ++i) {
        int live_i = 0;
        for (int h = 0; h < H; ++h) {
            const uint8_t o = ops[(size_t)i * H + h];
            if (o != D2FT_OP_SKIP) ++live_i;
            if (o == D2FT_OP_FULL) ops_union[h] = D2FT_OP_FULL;
            else if (o == D2FT_OP_FWD && ops_union[h] == D2FT_OP_SKIP) ops_union[h] = D2FT_OP_FWD;
        }
        if (live_i == 0) return false;   // that micro-batch's rows take no projection bias: per-micro-batch calls
    }
    int32_t live[D2FT_MAX_HEADS], nf = 0, nl = 0;
    if (compact(ops_union, H, live, &nf, &nl) != D2FT_OK) return false;
    memset(mask, 0, sizeof(*mask));
    mask->n = n_micro;
    mask->n_live_pos = nl;
    mask->n_full_pos = nf;
    int end = 0;
    for (int i = 0; i < n_micro; ++i) {
        end += mb_images[i];
        mask->img_end[i] = end;
        for (int p = 0; p < nl; ++p) {
            const uint8_t o = ops[(size_t)i * H + live[p]];
            if (o != D2FT_OP_SKIP) mask->live[i] |= 1ull << p;
            if (o == D2FT_OP_FULL) mask->full[i] |= 1ull << p;
        }
    }
    return true;
}

size_t d2ft_block_saved_bytes_mb(const d2ft_block_desc* desc, int32_t n_micro, const int32_t* mb_images) {
    d2ft_status why;
    if (!desc_ok(desc, &why) || !micro_ok(desc, n_micro, mb_images)) return 0;
    return micro_plan(desc, n_micro, mb_images).total;
}

d2ft_status d2ft_block_fwd_mb(const d2ft_block_desc* desc, const d2ft_block_weights* w, int32_t n_micro,
                              const int32_t* mb_images, const uint8_t* ops, const void* x, void* y, void* saved,
                              void* scratch, void* hip_stream) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!micro_ok(desc, n_micro, mb_images)) return mb_images ? D2FT_ESHAPE : D2FT_EINVAL;
    if (!weights_ok(desc, w) || !ops || !x || !y || !saved || !scratch || x == y) return D2FT_EINVAL;
    if (!aligned16(x) || !aligned16(y) || ((uintptr_t)saved & 255) || ((uintptr_t)scratch & 255)) return D2FT_EINVAL;
    for (int i = 0; i < n_micro * desc->heads; ++i)   // validate every code before the first launch
        if (ops[i] < D2FT_OP_FULL || ops[i] > D2FT_OP_SKIP) return D2FT_EINVAL;
    const MicroPlan P = micro_plan(desc, n_micro, mb_images);
    const size_t row_bytes = (size_t)desc->tokens * desc->width * elem_size(desc->dtype);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char* sv = static_cast<char*>(saved);
    if (n_micro == 1) return block_fwd_impl(desc, w, ops, x, y, sv, sv, scratch, st, PART_BOTH);   // the plain call
    {
        uint8_t ops_union[D2FT_MAX_HEADS];
        MicroMask mask;
        if (micro_union(desc, n_micro, mb_images, ops, ops_union, &mask))
            return block_fwd_impl(desc, w, ops_union, x, y, sv, sv, scratch, st, PART_BOTH, &mask);
    }
    size_t img0 = 0;
    for (int i = 0; i < n_micro; ++i) {
        d2ft_block_desc d = *desc;
        d.batch = mb_images[i];
        const char* xi = static_cast<const char*>(x) + img0 * row_bytes;
        // attention half alone: x1 of these images goes into the whole-batch x1
        void* out = P.shared_mlp ? (void*)(sv + P.x1 + img0 * row_bytes) : (void*)(static_cast<char*>(y) + img0 * row_bytes);
        const d2ft_status rc = block_fwd_impl(&d, w, ops + (size_t)i * desc->heads, xi, out, sv + P.at[i], sv + P.at[i],
                                              scratch, st, P.shared_mlp ? PART_ATTN : PART_BOTH);
        if (rc != D2FT_OK) return rc;
        img0 += mb_images[i];
    }
    if (P.shared_mlp) {
        const SavedLayout L = saved_layout(dims_of(desc));
        uint8_t any[D2FT_MAX_HEADS];   // op codes play no part in the ungated feed-forward half
        for (int h = 0; h < desc->heads; ++h) any[h] = D2FT_OP_FULL;
        return block_fwd_impl(desc, w, any, sv + P.x1, y, nullptr, sv + P.mlp - L.mean2, scratch, st, PART_MLP);
    }
    return D2FT_OK;
}

d2ft_status d2ft_block_bwd_mb(const d2ft_block_desc* desc, const d2ft_block_weights* w, int32_t n_micro,
                              const int32_t* mb_images, const uint8_t* ops, const void* x, const void* dy, void* dx,
                              const d2ft_block_grads* grads, const void* saved, void* scratch, void* hip_stream) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!micro_ok(desc, n_micro, mb_images)) return mb_images ? D2FT_ESHAPE : D2FT_EINVAL;
    if (!weights_ok(desc, w) || !ops || !x || !dy || !dx || !saved || !grads || !scratch || dy == dx) return D2FT_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || ((uintptr_t)saved & 255) || ((uintptr_t)scratch & 255))
        return D2FT_EINVAL;
    if (!grads_aligned(grads)) return D2FT_EINVAL;
    for (int i = 0; i < n_micro * desc->heads; ++i)
        if (ops[i] < D2FT_OP_FULL || ops[i] > D2FT_OP_SKIP) return D2FT_EINVAL;
    const MicroPlan P = micro_plan(desc, n_micro, mb_images);
    const size_t row_bytes = (size_t)desc->tokens * desc->width * elem_size(desc->dtype);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const char* sv = static_cast<const char*>(saved);
    if (n_micro == 1) return block_bwd_impl(desc, w, ops, x, dy, dx, grads, sv, sv, scratch, st, PART_BOTH);
    {
        uint8_t ops_union[D2FT_MAX_HEADS];
        MicroMask mask;
        if (micro_union(desc, n_micro, mb_images, ops, ops_union, &mask))
            return block_bwd_impl(desc, w, ops_union, x, dy, dx, grads, sv, sv, scratch, st, PART_BOTH, &mask);
    }
    if (P.shared_mlp) {   // feed-forward half over the whole batch: dx <- dx1, with the caller's flags
        const SavedLayout L = saved_layout(dims_of(desc));
        uint8_t any[D2FT_MAX_HEADS];
        for (int h = 0; h < desc->heads; ++h) any[h] = D2FT_OP_FULL;
        const d2ft_status rc = block_bwd_impl(desc, w, any, sv + P.x1, dy, dx, grads, nullptr, sv + P.mlp - L.mean2,
                                              scratch, st, PART_MLP);
        if (rc != D2FT_OK) return rc;
    }
    size_t img0 = 0;
    for (int i = 0; i < n_micro; ++i) {
        d2ft_block_desc d = *desc;
        d.batch = mb_images[i];
        if (i > 0) d.flags |= D2FT_FLAG_ACCUM_GRADS;   // later micro-batches add to the first one's result
        const char* xi = static_cast<const char*>(x) + img0 * row_bytes;
        char* dxi = static_cast<char*>(dx) + img0 * row_bytes;
        // attention half alone: dx1 of these images sits in dx and is rewritten in place
        const char* dyi = P.shared_mlp ? dxi : static_cast<const char*>(dy) + img0 * row_bytes;
        const d2ft_status rc = block_bwd_impl(&d, w, ops + (size_t)i * desc->heads, xi, dyi, dxi, grads, sv + P.at[i],
                                              sv + P.at[i], scratch, st, P.shared_mlp ? PART_ATTN : PART_BOTH);
        if (rc != D2FT_OK) return rc;
        img0 += mb_images[i];
    }
    return D2FT_OK;
}

// spans of the tensors one head owns; pointers may be NULL (then the span is dropped)
static ScoreArgs score_spans(const d2ft_block_desc* desc, const d2ft_block_weights* t) {
    const Dims s = dims_of(desc);
    const long D = s.D, H = s.H, r = s.r, Dm = s.Dm;
    const long S = (desc->flags & D2FT_FLAG_GATE_FFN) ? Dm / H : 0;
    ScoreArgs a;
    memset(&a, 0, sizeof(a));
    a.H = (int)H;
    auto add = [&](const void* p, bool present, long first, long head_stride, long rows, long cols, long stride) {
        if (!present) return;
        ScoreSpan& sp = a.span[a.n++];
        sp.p = p; sp.first = first; sp.head_stride = head_stride; sp.stride = stride;
        sp.rows = (int)rows; sp.cols8 = (int)(cols / 8);
        long n = (rows * cols / 8 + 1023) / 1024;   // about four 8-element pieces per thread
        sp.nchunks = (int)(n < 1 ? 1 : (n > 64 ? 64 : n));
        sp.chunk0 = a.total_chunks;
        a.total_chunks += sp.nchunks;
    };
    // with t == NULL every span counts (sizing the workspace)
    for (long p = 0; p < 3; ++p) {
        add(t ? t->w_qkv : nullptr, !t || t->w_qkv, p * H * 64 * D, 64 * D, 1, 64 * D, 64 * D);
        add(t ? t->b_qkv : nullptr, !t || t->b_qkv, p * H * 64, 64, 1, 64, 64);
    }
    add(t ? t->w_o : nullptr, !t || t->w_o, 0, 64, D, 64, H * 64);
    if (r > 0) {
        add(t ? t->lora_a_q : nullptr, !t || t->lora_a_q, 0, r * D, 1, r * D, r * D);
        add(t ? t->lora_a_v : nullptr, !t || t->lora_a_v, 0, r * D, 1, r * D, r * D);
        add(t ? t->lora_b_q : nullptr, !t || t->lora_b_q, 0, 64 * r, 1, 64 * r, 64 * r);
        add(t ? t->lora_b_v : nullptr, !t || t->lora_b_v, 0, 64 * r, 1, 64 * r, 64 * r);
    }
    if (S > 0) {
        add(t ? t->w1 : nullptr, !t || t->w1, 0, S * D, 1, S * D, S * D);
        add(t ? t->b1 : nullptr, !t || t->b1, 0, S, 1, S, S);
        add(t ? t->w2 : nullptr, !t || t->w2, 0, S, D, S, Dm);
    }
    return a;
}

size_t d2ft_scores_workspace_bytes(const d2ft_block_desc* desc) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return 0;
    const ScoreArgs a = score_spans(desc, nullptr);
    return align256((size_t)desc->heads * (a.total_chunks + 1) * sizeof(double));
}

d2ft_status d2ft_subnet_scores(const d2ft_block_desc* desc, const d2ft_block_weights* t, int32_t kind, double* scores_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!t || !scores_out || !workspace || ((uintptr_t)workspace & 255)) return D2FT_EINVAL;
    if (kind != D2FT_SCORE_FISHER && kind != D2FT_SCORE_MAGNITUDE) return D2FT_EINVAL;
    const size_t need = d2ft_scores_workspace_bytes(desc);
    if (need == 0 || workspace_bytes < need) return D2FT_ESHAPE;
    {
        const void* ps[] = {t->w_qkv, t->b_qkv, t->w_o, t->lora_a_q, t->lora_a_v, t->lora_b_q, t->lora_b_v, t->w1, t->b1, t->w2};
        for (const void* p : ps)
            if (p && !aligned16(p)) return D2FT_EINVAL;
    }
    const ScoreArgs a = score_spans(desc, t);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    {   // gradients or buffers an earlier backward call may still be working on
        const d2ft_status rj = join_pending(st);
        if (rj != D2FT_OK) return rj;
    }
    double* partial = static_cast<double*>(workspace);
    double* out = partial + (size_t)desc->heads * score_spans(desc, nullptr).total_chunks;
    if (a.n == 0) {
        for (int h = 0; h < desc->heads; ++h) scores_out[h] = 0.0;
        return D2FT_OK;
    }
    D2FT_TRY(launch_subnet_scores(desc->dtype, a, kind, partial, out, st));
    if (hipMemcpyAsync(scores_out, out, (size_t)desc->heads * sizeof(double), hipMemcpyDeviceToHost, st) != hipSuccess)
        return D2FT_EDEVICE;
    if (hipStreamSynchronize(st) != hipSuccess) return D2FT_EDEVICE;
    return D2FT_OK;
}

d2ft_status d2ft_sgd_step(const d2ft_block_desc* desc, const d2ft_block_grads* w, const d2ft_block_weights* g,
                          const d2ft_block_grads* v, const d2ft_block_grads* master, const uint8_t* ops,
                          const d2ft_sgd_params* prm, void* hip_stream) {
    d2ft_status why;
    if (!desc_ok(desc, &why)) return why;
    if (!w || !g || !v || !ops || !prm) return D2FT_EINVAL;
    if (!isfinite(prm->lr) || !isfinite(prm->momentum) || !isfinite(prm->weight_decay)) return D2FT_EINVAL;
    const Dims s = dims_of(desc);
    HeadList upd, one;
    upd.n = 0;
    one.n = 1; one.h[0] = 0;
    for (int h = 0; h < s.H; ++h) {
        if (ops[h] < D2FT_OP_FULL || ops[h] > D2FT_OP_SKIP) return D2FT_EINVAL;
        if (ops[h] == D2FT_OP_FULL) upd.h[upd.n++] = (uint8_t)h;
    }
    const long D = s.D, H = s.H, r = s.r, Dm = s.Dm;
    const bool gate = (desc->flags & D2FT_FLAG_GATE_FFN) != 0;
    const long S = gate ? Dm / H : 0;
    SgdArgs per_head, shared;
    memset(&per_head, 0, sizeof(per_head));
    memset(&shared, 0, sizeof(shared));
    per_head.lr = shared.lr = prm->lr;
    per_head.momentum = shared.momentum = prm->momentum;
    per_head.weight_decay = shared.weight_decay = prm->weight_decay;
    bool bad = false;
    auto add = [&](SgdArgs& a, void* wp, const void* gp, void* vp, void* mp, long first, long head_stride, long rows,
                   long cols, long stride) {
        if (!wp || !gp || !vp) return;
        if (!aligned16(wp) || !aligned16(gp) || !aligned16(vp) || (mp && !aligned16(mp))) { bad = true; return; }
        SgdSpan& sp = a.span[a.n++];
        sp.w = wp; sp.g = gp; sp.v = static_cast<float*>(vp); sp.master = static_cast<float*>(mp);
        sp.first = first; sp.head_stride = head_stride; sp.stride = stride;
        sp.rows = (int)rows; sp.cols8 = (int)(cols / 8);
        long n = (rows * cols / 8 + 511) / 512;   // about two 8-element pieces per thread
        sp.nchunks = (int)(n < 1 ? 1 : (n > 256 ? 256 : n));
        sp.chunk0 = a.total_chunks;
        a.total_chunks += sp.nchunks;
    };
#define D2FT_M(f) (master ? master->f : nullptr)
    for (long p = 0; p < 3; ++p) {
        add(per_head, w->w_qkv, g->w_qkv, v->w_qkv, D2FT_M(w_qkv), p * H * 64 * D, 64 * D, 1, 64 * D, 64 * D);
        add(per_head, w->b_qkv, g->b_qkv, v->b_qkv, D2FT_M(b_qkv), p * H * 64, 64, 1, 64, 64);
    }
    add(per_head, w->w_o, g->w_o, v->w_o, D2FT_M(w_o), 0, 64, D, 64, H * 64);
    if (r > 0) {
        add(per_head, w->lora_a_q, g->lora_a_q, v->lora_a_q, D2FT_M(lora_a_q), 0, r * D, 1, r * D, r * D);
        add(per_head, w->lora_a_v, g->lora_a_v, v->lora_a_v, D2FT_M(lora_a_v), 0, r * D, 1, r * D, r * D);
        add(per_head, w->lora_b_q, g->lora_b_q, v->lora_b_q, D2FT_M(lora_b_q), 0, 64 * r, 1, 64 * r, 64 * r);
        add(per_head, w->lora_b_v, g->lora_b_v, v->lora_b_v, D2FT_M(lora_b_v), 0, 64 * r, 1, 64 * r, 64 * r);
    }
    SgdArgs& ffn = gate ? per_head : shared;
    add(ffn, w->w1, g->w1, v->w1, D2FT_M(w1), 0, gate ? S * D : 0, 1, gate ? S * D : Dm * D, gate ? S * D : Dm * D);
    add(ffn, w->b1, g->b1, v->b1, D2FT_M(b1), 0, gate ? S : 0, 1, gate ? S : Dm, gate ? S : Dm);
    add(ffn, w->w2, g->w2, v->w2, D2FT_M(w2), 0, gate ? S : 0, gate ? D : 1, gate ? S : D * Dm, gate ? Dm : D * Dm);
    add(shared, w->ln1_g, g->ln1_g, v->ln1_g, D2FT_M(ln1_g), 0, 0, 1, D, D);
    add(shared, w->ln1_b, g->ln1_b, v->ln1_b, D2FT_M(ln1_b), 0, 0, 1, D, D);
    add(shared, w->b_o, g->b_o, v->b_o, D2FT_M(b_o), 0, 0, 1, D, D);
    add(shared, w->ln2_g, g->ln2_g, v->ln2_g, D2FT_M(ln2_g), 0, 0, 1, D, D);
    add(shared, w->ln2_b, g->ln2_b, v->ln2_b, D2FT_M(ln2_b), 0, 0, 1, D, D);
    add(shared, w->b2, g->b2, v->b2, D2FT_M(b2), 0, 0, 1, D, D);
#undef D2FT_M
    if (bad) return D2FT_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    {   // gradients or buffers an earlier backward call may still be working on
        const d2ft_status rj = join_pending(st);
        if (rj != D2FT_OK) return rj;
    }
    D2FT_TRY(launch_sgd(s.dtype, per_head, upd, st));
    D2FT_TRY(launch_sgd(s.dtype, shared, one, st));
    return D2FT_OK;
}

// ---- the two subnets outside the blocks ----
struct EmbedLayout {
    long rows, K;          // B * patches per image, C * P * P
    int Np;
    size_t proj, dproj, part, colpart, total;
};
static bool embed_ok(const d2ft_embed_desc* d) {
    if (!d) return false;
    if (d->dtype != D2FT_F32 && d->dtype != D2FT_BF16) return false;
    if (d->batch < 1 || d->channels < 1 || d->patch < 8 || d->patch % 8) return false;
    if (d->height < d->patch || d->width_px < d->patch || d->height % d->patch || d->width_px % d->patch) return false;
    if (d->width < 8 || d->width % 8) return false;
    const long np = (long)(d->height / d->patch) * (d->width_px / d->patch);
    if (np > 4096 || (long)d->batch * np > (1L << 24)) return false;
    if ((long)d->channels * d->patch * d->patch > 65536) return false;
    return true;
}
static EmbedLayout embed_layout(const d2ft_embed_desc* d) {
    EmbedLayout L;
    L.Np = (d->height / d->patch) * (d->width_px / d->patch);
    L.rows = (long)d->batch * L.Np;
    L.K = (long)d->channels * d->patch * d->patch;
    const size_t es = elem_size(d->dtype);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off += align256(bytes); return at; };
    L.proj = take((size_t)L.rows * d->width * es);
    L.dproj = take((size_t)L.rows * d->width * es);
    L.part = take((size_t)kMaxSplits * d->width * L.K * 4);
    L.colpart = take((size_t)kColChunks * d->width * 4);
    L.total = off;
    return L;
}
// a block descriptor that carries dtype and flags to the GEMM helpers
static d2ft_block_desc helper_desc(int dtype, uint32_t flags) {
    d2ft_block_desc b;
    memset(&b, 0, sizeof(b));
    b.dtype = dtype;
    b.flags = flags;
    return b;
}

size_t d2ft_embed_saved_bytes(const d2ft_embed_desc* d) {
    if (!embed_ok(d)) return 0;
    const EmbedLayout L = embed_layout(d);
    return align256((size_t)L.rows * L.K * elem_size(d->dtype));
}
size_t d2ft_embed_scratch_bytes(const d2ft_embed_desc* d) {
    if (!embed_ok(d)) return 0;
    return embed_layout(d).total;
}

d2ft_status d2ft_patch_embed_fwd(const d2ft_embed_desc* d, const void* images, const void* w_pe, const void* b_pe,
                                 const void* cls, const void* pos, void* tokens, void* saved, void* scratch,
                                 void* hip_stream) {
    if (!d) return D2FT_EINVAL;
    if (!embed_ok(d)) return D2FT_ESHAPE;
    if (!images || !w_pe || !b_pe || !cls || !pos || !tokens || !saved || !scratch) return D2FT_EINVAL;
    const void* ps[] = {images, w_pe, b_pe, cls, pos, tokens};
    for (const void* p : ps)
        if (!aligned16(p)) return D2FT_EINVAL;
    if (((uintptr_t)saved & 255) || ((uintptr_t)scratch & 255)) return D2FT_EINVAL;
    const EmbedLayout L = embed_layout(d);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    {   // gradients or buffers an earlier backward call may still be working on
        const d2ft_status rj = join_pending(st);
        if (rj != D2FT_OK) return rj;
    }
    char* ws = static_cast<char*>(scratch);
    D2FT_TRY(launch_im2col(d->dtype, images, saved, d->batch, d->channels, d->height, d->width_px, d->patch, st));
    const d2ft_block_desc hd = helper_desc(d->dtype, d->flags);
    GemmArgs g = gemm_base();
    g.A = saved; g.a_rs = L.K; g.a_cs = 1;
    g.B = w_pe; g.b_rs = 1; g.b_cs = L.K;
    g.M = (int)L.rows; g.N = d->width; g.K = (int)L.K;
    g.C = ws + L.proj; g.ldc = d->width;
    g.bias = b_pe;
    D2FT_TRY_UNTIMED(run_gemm(g, &hd, st));
    D2FT_TRY(launch_assemble_tokens(d->dtype, ws + L.proj, cls, pos, tokens, d->batch, L.Np, d->width, st));
    return D2FT_OK;
}

d2ft_status d2ft_patch_embed_bwd(const d2ft_embed_desc* d, const void* dtokens, void* g_w_pe, void* g_b_pe, void* g_cls,
                                 void* g_pos, const void* saved, void* scratch, void* hip_stream) {
    if (!d) return D2FT_EINVAL;
    if (!embed_ok(d)) return D2FT_ESHAPE;
    if (!dtokens || !saved || !scratch || !aligned16(dtokens)) return D2FT_EINVAL;
    const void* ps[] = {g_w_pe, g_b_pe, g_cls, g_pos};
    for (const void* p : ps)
        if (p && !aligned16(p)) return D2FT_EINVAL;
    if (((uintptr_t)saved & 255) || ((uintptr_t)scratch & 255)) return D2FT_EINVAL;
    const EmbedLayout L = embed_layout(d);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    {   // gradients or buffers an earlier backward call may still be working on
        const d2ft_status rj = join_pending(st);
        if (rj != D2FT_OK) return rj;
    }
    char* ws = static_cast<char*>(scratch);
    const int accum = (d->flags & D2FT_FLAG_ACCUM_GRADS) ? 1 : 0;
    D2FT_TRY(launch_embed_bwd_gather(d->dtype, dtokens, ws + L.dproj, g_pos, g_cls, d->batch, L.Np, d->width, accum, st));
    const d2ft_block_desc hd = helper_desc(d->dtype, d->flags);
    Dims s;
    memset(&s, 0, sizeof(s));
    s.M = L.rows; s.dtype = d->dtype; s.es = elem_size(d->dtype); s.D = d->width;
    Remap64 none;
    memset(&none, 0, sizeof(none));
    if (g_w_pe) {   // dW_pe = dproj^T patches
        const d2ft_status rc = weight_grad(&hd, s, ws + L.dproj, d->width, saved, L.K, d->width, (int)L.K,
                                           (float*)(ws + L.part), g_w_pe, L.K, RED_REMAP_NONE, none, st);
        if (rc != D2FT_OK) return rc;
    }
    if (g_b_pe) {
        ColReduceBatch batch;
        memset(&batch, 0, sizeof(batch));
        d2ft_status rc = bias_grad(s, ws + L.dproj, d->width, d->width, (float*)(ws + L.colpart), g_b_pe, 0, &batch, st);
        if (rc != D2FT_OK) return rc;
        rc = flush_bias_grads(&hd, s, &batch, none, none, st);
        if (rc != D2FT_OK) return rc;
    }
    return D2FT_OK;
}

struct HeadLayout {
    size_t xhat, h, dh, rstd, logits, dl, loss_b, loss, labels, total;
};
static bool head_ok(const d2ft_head_desc* d) {
    if (!d) return false;
    if (d->dtype != D2FT_F32 && d->dtype != D2FT_BF16) return false;
    if (d->batch < 1 || d->batch > 65536 || d->tokens < 1 || d->tokens > 4097) return false;
    if (d->width < 8 || d->width % 8 || d->width > 16384) return false;
    if (d->classes < 1 || d->classes > 65536) return false;
    if (!(d->ln_eps > 0.0f) || !isfinite(d->ln_eps)) return false;
    return true;
}
static HeadLayout head_layout(const d2ft_head_desc* d) {
    HeadLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off += align256(bytes); return at; };
    const size_t B = d->batch, D = d->width, n = d->classes;
    L.xhat = take(B * D * 4); L.h = take(B * D * 4); L.dh = take(B * D * 4); L.rstd = take(B * 4);
    L.logits = take(B * n * 4); L.dl = take(B * n * 4); L.loss_b = take(B * 4); L.loss = take(4);
    L.labels = take(B * 4);
    L.total = off;
    return L;
}
size_t d2ft_head_scratch_bytes(const d2ft_head_desc* d) { return head_ok(d) ? head_layout(d).total : 0; }

d2ft_status d2ft_classifier_fwd_bwd(const d2ft_head_desc* d, const void* tokens, const void* ln_g, const void* ln_b,
                                    const void* w_c, const void* b_c, const int32_t* labels, float* loss_out, void* dtokens,
                                    void* g_ln_g, void* g_ln_b, void* g_w_c, void* g_b_c, void* scratch, void* hip_stream) {
    if (!d) return D2FT_EINVAL;
    if (!head_ok(d)) return D2FT_ESHAPE;
    if (!tokens || !ln_g || !ln_b || !w_c || !b_c || !labels || !loss_out || !dtokens || !scratch) return D2FT_EINVAL;
    if (((uintptr_t)scratch & 255) || tokens == dtokens) return D2FT_EINVAL;
    for (int b = 0; b < d->batch; ++b)
        if (labels[b] < 0 || labels[b] >= d->classes) return D2FT_EINVAL;
    const HeadLayout L = head_layout(d);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    {   // gradients or buffers an earlier backward call may still be working on
        const d2ft_status rj = join_pending(st);
        if (rj != D2FT_OK) return rj;
    }
    char* ws = static_cast<char*>(scratch);
    if (hipMemcpyAsync(ws + L.labels, labels, (size_t)d->batch * 4, hipMemcpyHostToDevice, st) != hipSuccess)
        return D2FT_EDEVICE;
    D2FT_TRY(launch_classifier(d->dtype, tokens, ln_g, ln_b, w_c, b_c, (const int32_t*)(ws + L.labels), d->batch, d->tokens,
                               d->width, d->classes, d->ln_eps, (float*)(ws + L.xhat), (float*)(ws + L.h),
                               (float*)(ws + L.rstd), (float*)(ws + L.logits), (float*)(ws + L.dl), (float*)(ws + L.loss_b),
                               (float*)(ws + L.dh), dtokens, g_w_c, g_b_c, g_ln_g, g_ln_b, (float*)(ws + L.loss),
                               (d->flags & D2FT_FLAG_ACCUM_GRADS) ? 1 : 0, st));
    if (hipMemcpyAsync(loss_out, ws + L.loss, 4, hipMemcpyDeviceToHost, st) != hipSuccess) return D2FT_EDEVICE;
    if (hipStreamSynchronize(st) != hipSuccess) return D2FT_EDEVICE;
    return D2FT_OK;
}

size_t d2ft_knapsack_workspace_bytes(int32_t n_knapsacks, int32_t n_items, const int32_t* cap_full,
                                     const int32_t* cap_fwd) {
    if (n_knapsacks < 1 || n_items < 1 || !cap_full || !cap_fwd) return 0;
    long cmax = 0;
    for (int k = 0; k < n_knapsacks; ++k) {
        if (cap_full[k] < 0 || cap_fwd[k] < 0) return 0;
        if (cap_full[k] > cmax) cmax = cap_full[k];
        if (cap_fwd[k] > cmax) cmax = cap_fwd[k];
    }
    const size_t stride = align256((size_t)cmax + 1);
    const size_t probs = (size_t)n_knapsacks * 2;
    size_t total = 0;
    total += align256((size_t)n_knapsacks * n_items * 8) * 2;   // scores
    total += align256((size_t)n_knapsacks * 4) * 4;             // costs, capacities
    total += align256(probs * 2 * stride * 8);                  // two table rows per problem
    total += align256(probs * n_items * stride);                // change flags
    total += align256(probs * n_items);                         // 0/1 selections
    total += align256((size_t)n_knapsacks * n_items);           // merged codes
    return total;
}

// validation and launch sequence shared by the two knapsack entry points; `workspace` is device memory
static d2ft_status knapsack_run(int32_t n_knapsacks, int32_t n_items, const double* score_full,
                                const double* score_fwd, const int32_t* cost_fwd, const int32_t* cost_bwd,
                                const int32_t* cap_full, const int32_t* cap_fwd, uint8_t* ops_out, void* workspace,
                                size_t workspace_bytes, hipStream_t st) {
    if (!score_full || !score_fwd || !cost_fwd || !cost_bwd || !cap_full || !cap_fwd || !ops_out || !workspace)
        return D2FT_EINVAL;
    if (n_knapsacks < 1 || n_items < 1) return D2FT_ESHAPE;
    if ((uintptr_t)workspace & 255) return D2FT_EINVAL;
    long cmax = 0;
    for (int k = 0; k < n_knapsacks; ++k) {
        if (cost_fwd[k] < 1 || cost_bwd[k] < 0 || cap_full[k] < 0 || cap_fwd[k] < 0) return D2FT_EINVAL;
        if ((long)cost_fwd[k] + cost_bwd[k] > 0x3fffffff) return D2FT_EINVAL;
        if (cap_full[k] > cmax) cmax = cap_full[k];
        if (cap_fwd[k] > cmax) cmax = cap_fwd[k];
    }
    const size_t nsc = (size_t)n_knapsacks * n_items;
    for (size_t i = 0; i < nsc; ++i)
        if (!isfinite(score_full[i]) || !isfinite(score_fwd[i])) return D2FT_EINVAL;
    const size_t need = d2ft_knapsack_workspace_bytes(n_knapsacks, n_items, cap_full, cap_fwd);
    if (need == 0 || workspace_bytes < need) return D2FT_ESHAPE;

    char* ws = static_cast<char*>(workspace);
    size_t off = 0;
    auto take = [&](size_t bytes) { char* at = ws + off; off += align256(bytes); return at; };
    const size_t stride = align256((size_t)cmax + 1);
    const size_t probs = (size_t)n_knapsacks * 2;
    KnapsackArgs a;
    a.n_knapsacks = n_knapsacks; a.n_items = n_items; a.stride = (long)stride;
    double* d_sf = (double*)take(nsc * 8);
    double* d_so = (double*)take(nsc * 8);
    int* d_cf = (int*)take((size_t)n_knapsacks * 4);
    int* d_cb = (int*)take((size_t)n_knapsacks * 4);
    int* d_capf = (int*)take((size_t)n_knapsacks * 4);
    int* d_capo = (int*)take((size_t)n_knapsacks * 4);
    a.rows = (double*)take(probs * 2 * stride * 8);
    a.changed = (uint8_t*)take(probs * n_items * stride);
    a.selected = (uint8_t*)take(probs * n_items);
    uint8_t* d_ops = (uint8_t*)take(nsc);
    a.score_full = d_sf; a.score_fwd = d_so; a.cost_fwd = d_cf; a.cost_bwd = d_cb; a.cap_full = d_capf; a.cap_fwd = d_capo;

    D2FT_TRY(hipMemcpyAsync(d_sf, score_full, nsc * 8, hipMemcpyHostToDevice, st));
    D2FT_TRY(hipMemcpyAsync(d_so, score_fwd, nsc * 8, hipMemcpyHostToDevice, st));
    D2FT_TRY(hipMemcpyAsync(d_cf, cost_fwd, (size_t)n_knapsacks * 4, hipMemcpyHostToDevice, st));
    D2FT_TRY(hipMemcpyAsync(d_cb, cost_bwd, (size_t)n_knapsacks * 4, hipMemcpyHostToDevice, st));
    D2FT_TRY(hipMemcpyAsync(d_capf, cap_full, (size_t)n_knapsacks * 4, hipMemcpyHostToDevice, st));
    D2FT_TRY(hipMemcpyAsync(d_capo, cap_fwd, (size_t)n_knapsacks * 4, hipMemcpyHostToDevice, st));
    D2FT_TRY(launch_knapsack(a, d_ops, st));
    D2FT_TRY(hipMemcpyAsync(ops_out, d_ops, nsc, hipMemcpyDeviceToHost, st));
    D2FT_TRY(hipStreamSynchronize(st));
    return D2FT_OK;
}

d2ft_status d2ft_select_knapsack(int32_t n_knapsacks, int32_t n_items, const double* score_full,
                                 const double* score_fwd, const int32_t* cost_fwd, const int32_t* cost_bwd,
                                 const int32_t* cap_full, const int32_t* cap_fwd, uint8_t* ops_out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
    return knapsack_run(n_knapsacks, n_items, score_full, score_fwd, cost_fwd, cost_bwd, cap_full, cap_fwd, ops_out,
                        workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

// ---- the knapsack selection for callers that cannot allocate ----
// Its workspace is a file-scope device array.  Every GPU the library runs on holds its own copy of the
// array at its own address for the life of the process; the address is looked up once per device, with
// that device current, and host code uses that pointer - never the array's name, which on the host is only
// a handle for the lookup.
static __device__ __align__(256) unsigned char scratch[D2FT_KNAPSACK_STATIC_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // per device, NULL until the first call on it

size_t d2ft_knapsack_static_bytes(void) { return sizeof(scratch); }

d2ft_status d2ft_select_knapsack_static(int32_t n_knapsacks, int32_t n_items, const double* score_full,
                                        const double* score_fwd, const int32_t* cost_fwd, const int32_t* cost_bwd,
                                        const int32_t* cap_full, const int32_t* cap_fwd, uint8_t* ops_out,
                                        void* hip_stream) {
    if (!cap_full || !cap_fwd) return D2FT_EINVAL;
    if (n_knapsacks < 1 || n_items < 1) return D2FT_ESHAPE;
    for (int k = 0; k < n_knapsacks; ++k)
        if (cap_full[k] < 0 || cap_fwd[k] < 0) return D2FT_EINVAL;
    // a problem beyond the array's size is refused before anything touches the device
    const size_t need = d2ft_knapsack_workspace_bytes(n_knapsacks, n_items, cap_full, cap_fwd);
    if (need == 0 || need > sizeof(scratch)) return D2FT_ESHAPE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return D2FT_EDEVICE;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return D2FT_EDEVICE;
        g_scratch_ptr[dev] = ptr;
    }
    // nothing in the workspace has to start at zero: the kernel initialises the table row, the selection
    // flags and every change flag it later reads, so what the previous call left behind is harmless
    return knapsack_run(n_knapsacks, n_items, score_full, score_fwd, cost_fwd, cost_bwd, cap_full, cap_fwd, ops_out,
                        g_scratch_ptr[dev], sizeof(scratch), static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
