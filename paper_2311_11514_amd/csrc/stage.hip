// Host runtime behind the C ABI of include/hexgen.h: argument validation, shard slicing and
// repacking of the weights, the KV-cache object, the reusable activation workspace (the paper's
// memory model, Appendix B "Model the memory constraint", counts a handful of activation buffers
// reused by all layers; the same idea here), and the per-layer launch sequence.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/hexgen.h"
#include "../../include/hexgen_bench.h"
#include "kernels.h"

#define HX_HIP(expr)                                                          \
    do {                                                                      \
        hipError_t e_ = (expr);                                               \
        if (e_ != hipSuccess) {                                               \
            (void)hipGetLastError();                                          \
            return e_ == hipErrorOutOfMemory ? HEXGEN_ERR_OOM : HEXGEN_ERR_DEVICE; \
        }                                                                     \
    } while (0)
#define HX_TRY(expr)                              \
    do {                                          \
        hexgen_status_t s_ = (expr);              \
        if (s_ != HEXGEN_OK) return s_;           \
    } while (0)

namespace {

constexpr int kDecodeMaxRows = 32;      // rows handled by the weight-streaming decode kernels
constexpr int kAttnRows = 128;            // new rows per block of the prefill attention (4 waves x 32)
constexpr int kMaxAttnSplit = 32;         // blocks per (sequence, kv head) the workspace has partials for
constexpr int kStaticAttnSplit = 8;       // what pick_attn_split chooses at most, and what the static scratch is laid out for

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

struct Layer {
    float *g_attn = nullptr, *g_ffn = nullptr;
    void *wqkv = nullptr, *wo = nullptr, *w13 = nullptr, *w2 = nullptr;
    bool loaded = false;
};

// Optional per-slot timing with HIP events recorded on the caller's stream (measurement surface).
enum { PROF_QKV = 0, PROF_WO = 1, PROF_W13 = 2, PROF_W2 = 3, PROF_ATTN = 4, PROF_CALL = 5, PROF_W13_MAIN = 6, PROF_SLOTS = 7 };
struct Profiler {
    unsigned mask = 0;                          // bit i set: slot i is timed
    std::vector<hipEvent_t> ev[PROF_SLOTS];     // start, stop, start, stop, ...
    void mark(int slot, hipStream_t s) {
        if (!(mask >> slot & 1u)) return;
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        (void)hipEventRecord(e, s);
        ev[slot].push_back(e);
    }
    void clear() {
        for (auto &v : ev) {
            for (hipEvent_t e : v) (void)hipEventDestroy(e);
            v.clear();
        }
    }
};

struct Workspace {
    int cap_rows = 0;
    float *h = nullptr;        // residual stream [T][H] fp32
    float *part = nullptr;     // projection outputs / split-K partials, fp32
    float *p32 = nullptr;      // reduced partial [T][H] fp32
    // bf16 path
    h16_t *n = nullptr, *o = nullptr, *u = nullptr, *q = nullptr;
    float *dec_part = nullptr;       // split partial sums of the batched decode projections
    size_t dec_part_floats = 0;
    float *gemm_part = nullptr;      // fp32 partial tiles of a split prefill contraction (short prompts)
    size_t gemm_part_floats = 0;
    h16_t *xa_n = nullptr, *xa_o = nullptr, *xa_u = nullptr;   // decode operands, compact hi/lo layout [32][K][2]
    h16_t *q_lo = nullptr;
    float *att_o = nullptr, *att_ml = nullptr;
    unsigned int *att_arrived = nullptr;      // per (sequence, kv head): split blocks that have finished; zero between launches
    float *ssq = nullptr;                       // decode: 2 x [H/16 units][DEC_SSQ_STRIDE] sums of squares
    float *ssq_pf = nullptr;                    // prefill: 2 x [H/128][T] sums of squares
    // fp32 path
    float *n32 = nullptr, *q32 = nullptr, *o32 = nullptr, *u32 = nullptr;
    // row bookkeeping
    int32_t *rowmap = nullptr;       // one block: row_seq | row_pos | cu_rows | pos0, packed by the sizes of the call
    int32_t *row_seq = nullptr, *row_pos = nullptr, *cu_rows = nullptr, *pos0 = nullptr;   // views into rowmap
    int32_t *items = nullptr;        // view into rowmap: the prefill attention's work list, (sequence, 128-row block) pairs
    int32_t *host_stage = nullptr;   // pinned staging for the arrays above
    int host_stage_cap = 0;
};

}  // namespace

struct hexgen_stage {
    int H, hq, hkv, F, L, t, r;
    int d, hq_l, hkv_l, F_l, nqkv, qw;     // qw = hq_l * d
    hexgen_dtype_t dtype;
    float eps = 1e-5f, theta = 10000.0f;
    std::vector<Layer> layers;
    std::vector<void *> taps;
    Workspace ws;
    Workspace *cur = nullptr;        // the workspace the decode flow runs on: &ws, or a view of the static scratch array
    int last_decode_rows = 0;        // rows of the last decode call that ran on the weight-streaming kernels
    int ws_batch_cap = 0;
    int64_t weight_bytes = 0;
    Profiler prof;
};

struct hexgen_kv_cache {
    hexgen_stage *st;
    int max_batch, max_seq, smax;          // smax = max_seq rounded up to 32
    void *k = nullptr, *v = nullptr;       // [L][max_batch][hkv_l][smax][d]
    int64_t layer_stride;                  // elements
    float *cos_tab = nullptr, *sin_tab = nullptr;   // [smax][d/2]
    float rope_theta_built = 0.f;
    std::vector<int32_t> lens;             // committed lengths (host copy)
    int32_t *d_lens = nullptr;
    int batch = 0;
    bool prefilled = false;
    int steps = 0;
};

namespace {

size_t esize(hexgen_dtype_t dt) { return dt == HEXGEN_F32 ? 4 : 2; }
bool is_h16(hexgen_dtype_t dt) { return dt == HEXGEN_BF16 || dt == HEXGEN_F16; }
bool known_dtype(hexgen_dtype_t dt) { return dt == HEXGEN_F32 || is_h16(dt); }
// The 16-bit kernels exist once per element type (namespaces bf16 and f16): pick by the stage's type.
#define HX_K(dt, fn, ...) ((dt) == HEXGEN_F16 ? f16::fn(__VA_ARGS__) : bf16::fn(__VA_ARGS__))

void free_ws(Workspace &w) {
    void *ptrs[] = {w.dec_part, w.gemm_part, w.h, w.part, w.p32, w.n, w.o, w.u, w.q, w.xa_n, w.xa_o, w.xa_u, w.q_lo, w.ssq, w.ssq_pf, w.att_o, w.att_ml, w.att_arrived, w.n32, w.q32, w.o32, w.u32,
                    w.rowmap};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (w.host_stage) (void)hipHostFree(w.host_stage);
    w = Workspace();
}

template <typename T>
hexgen_status_t dmalloc(T **p, size_t count) {
    *p = nullptr;
    if (count == 0) count = 1;
    HX_HIP(hipMalloc(reinterpret_cast<void **>(p), count * sizeof(T)));
    return HEXGEN_OK;
}

// (re)allocate the workspace for `rows` token rows and `batch` sequences
hexgen_status_t ensure_workspace(hexgen_stage *st, int rows, int batch) {
    Workspace &w = st->ws;
    if (rows <= w.cap_rows && batch <= st->ws_batch_cap) return HEXGEN_OK;
    HX_HIP(hipDeviceSynchronize());
    rows = std::max(rows, w.cap_rows);
    batch = std::max(batch, st->ws_batch_cap);
    free_ws(w);
    st->ws_batch_cap = 0;
    const size_t T = (size_t)rows, T16 = (size_t)round_up(rows, 16);
    const size_t nmax = (size_t)std::max(std::max(st->nqkv, st->H), 2 * st->F_l);
    HX_TRY(dmalloc(&w.h, (size_t)round_up(rows, 32) * st->H));
    if (st->dtype == HEXGEN_F32) {
        HX_TRY(dmalloc(&w.part, T * nmax));
        HX_TRY(dmalloc(&w.p32, T * st->H));
    }
    if (is_h16(st->dtype)) {
        HX_TRY(dmalloc(&w.n, T16 * st->H));
        HX_TRY(dmalloc(&w.o, T16 * st->qw));
        HX_TRY(dmalloc(&w.u, T16 * st->F_l));
        HX_TRY(dmalloc(&w.q, T16 * st->qw));
        const size_t drows = (size_t)std::min(rows, kDecodeMaxRows);
        HX_TRY(dmalloc(&w.xa_n, 2 * drows * st->H));
        HX_TRY(dmalloc(&w.xa_o, 2 * drows * st->qw));
        HX_TRY(dmalloc(&w.xa_u, 2 * drows * st->F_l));
        HX_TRY(dmalloc(&w.q_lo, drows * st->qw));
        if (drows > 2) {      // splits x features stays near 512 x 128 (see launch_splitk), plus one unsplit matrix
            w.dec_part_floats = drows * ((size_t)512 * 128 + 2 * nmax);
            HX_TRY(dmalloc(&w.dec_part, w.dec_part_floats));
        }
        w.gemm_part_floats = (size_t)16 << 20;      // 64 MB: 8 splits of the widest short-prompt launch
        HX_TRY(dmalloc(&w.gemm_part, w.gemm_part_floats));
        HX_TRY(dmalloc(&w.att_o, drows * st->hq_l * kMaxAttnSplit * st->d));
        HX_TRY(dmalloc(&w.att_ml, drows * st->hq_l * kMaxAttnSplit * 2));
        HX_TRY(dmalloc(&w.att_arrived, drows * st->hkv_l));
        HX_HIP(hipMemset(w.att_arrived, 0, drows * st->hkv_l * sizeof(unsigned int)));
        const size_t ssq_n = 2 * (size_t)(st->H / 16) * DEC_SSQ_STRIDE;
        HX_TRY(dmalloc(&w.ssq, ssq_n));
        HX_TRY(dmalloc(&w.ssq_pf, 2 * (size_t)(st->H / GEMM_SSQ_COLS + 1) * T));
        HX_HIP(hipMemset(w.ssq, 0, ssq_n * sizeof(float)));
        // padded rows of the packed operands are read by the GEMM tiles: keep them finite
        HX_HIP(hipMemset(w.n, 0, T16 * st->H * sizeof(h16_t)));
        HX_HIP(hipMemset(w.o, 0, T16 * st->qw * sizeof(h16_t)));
        HX_HIP(hipMemset(w.u, 0, T16 * st->F_l * sizeof(h16_t)));
    } else {
        HX_TRY(dmalloc(&w.n32, T * st->H));
        HX_TRY(dmalloc(&w.q32, T * st->qw));
        HX_TRY(dmalloc(&w.o32, T * st->qw));
        HX_TRY(dmalloc(&w.u32, T * st->F_l));
    }
    // row_seq, row_pos, cu_rows, pos0, new lengths, attention work list (at most rows / 128 + batch pairs)
    w.host_stage_cap = 2 * rows + 3 * batch + 1 + 2 * (rows / kAttnRows + batch);
    HX_TRY(dmalloc(&w.rowmap, (size_t)w.host_stage_cap));
    HX_HIP(hipHostMalloc(reinterpret_cast<void **>(&w.host_stage), (size_t)w.host_stage_cap * sizeof(int32_t),
                         hipHostMallocDefault));
    w.cap_rows = rows;
    st->ws_batch_cap = batch;
    // the zero fills above ran on the null stream; the caller's stream may be a non-blocking one that does not
    // order itself behind it
    HX_HIP(hipDeviceSynchronize());
    return HEXGEN_OK;
}

struct Rows {
    int T = 0, batch = 0, max_new = 0, n_items = 0;
    bool decode = false;
    RowMap rm{};
};

// Validate the new rows against the cache and build the device row maps.
hexgen_status_t setup_rows(hexgen_stage *st, hexgen_kv_cache *kv, const int32_t *seq_lens, int batch,
                           bool allow_decode, hipStream_t s, Rows *out) {
    if (batch <= 0) return HEXGEN_ERR_INVALID_ARG;
    if (batch > kv->max_batch) return HEXGEN_ERR_CAPACITY;
    Rows r;
    r.batch = batch;
    long total = 0;
    for (int i = 0; i < batch; ++i) {
        const int n = seq_lens ? seq_lens[i] : 1;
        if (n < 1) return HEXGEN_ERR_INVALID_ARG;
        if ((long)kv->lens[i] + n > kv->max_seq) return HEXGEN_ERR_CAPACITY;
        total += n;
        r.max_new = std::max(r.max_new, n);
    }
    if (total > 0x3fffffff) return HEXGEN_ERR_CAPACITY;
    r.T = (int)total;
    r.decode = allow_decode && r.max_new == 1 && r.T <= kDecodeMaxRows;
    HX_TRY(ensure_workspace(st, r.T, batch));
    Workspace &w = st->ws;
    w.row_seq = w.rowmap;
    w.row_pos = w.rowmap + r.T;
    w.cu_rows = w.rowmap + 2 * (size_t)r.T;
    w.pos0 = w.cu_rows + batch + 1;
    r.rm.row_seq = w.row_seq;
    r.rm.row_pos = w.row_pos;
    if (r.decode && is_h16(st->dtype)) {
        // the decode prologue kernel publishes row positions from the committed lengths on the device
    } else if (r.decode) {
        launch_decode_rowmap(kv->d_lens, w.row_seq, w.row_pos, batch, s);
    } else {
        // the pinned staging buffer may still feed an earlier async copy on this stream
        HX_HIP(hipStreamSynchronize(s));
        int32_t *hs = w.host_stage;
        int32_t *h_seq = hs, *h_pos = hs + r.T, *h_cu = hs + 2 * r.T, *h_p0 = h_cu + batch + 1;
        int row = 0;
        for (int i = 0; i < batch; ++i) {
            const int n = seq_lens ? seq_lens[i] : 1;
            h_cu[i] = row;
            h_p0[i] = kv->lens[i];
            for (int jn = 0; jn < n; ++jn, ++row) { h_seq[row] = i; h_pos[row] = kv->lens[i] + jn; }
        }
        h_cu[batch] = row;
        // The prefill attention's work list: one entry per (sequence, block of 128 new rows), the longest walks over
        // the cache first.  A ragged batch thus launches no empty blocks (a grid over the longest prompt's blocks
        // would: 45 % of it at lengths 128..4096) and its long walks do not end up alone at the tail of the launch.
        const size_t items_off = 2 * (size_t)r.T + 3 * (size_t)batch + 1;
        int32_t *h_items = hs + items_off;
        int n_items = 0;
        try {
            std::vector<std::pair<int, int>> order;         // (-last position of the block, index)
            for (int i = 0; i < batch; ++i) {
                const int n = seq_lens ? seq_lens[i] : 1;
                for (int rb = 0; rb * kAttnRows < n; ++rb, ++n_items) {
                    h_items[2 * n_items] = i;
                    h_items[2 * n_items + 1] = rb;
                    order.emplace_back(-(kv->lens[i] + std::min((rb + 1) * kAttnRows, n)), n_items);
                }
            }
            std::stable_sort(order.begin(), order.end());
            std::vector<int32_t> sorted(2 * (size_t)n_items);
            for (int k = 0; k < n_items; ++k) {
                sorted[2 * k] = h_items[2 * order[k].second];
                sorted[2 * k + 1] = h_items[2 * order[k].second + 1];
            }
            std::copy(sorted.begin(), sorted.end(), h_items);
        } catch (...) {                                     // no exception crosses the C boundary
            return HEXGEN_ERR_OOM;
        }
        r.n_items = n_items;
        w.items = w.rowmap + items_off;
        // host staging and device block share one packing: a single copy moves all the arrays
        HX_HIP(hipMemcpyAsync(w.rowmap, hs, sizeof(int32_t) * (items_off + 2 * (size_t)n_items), hipMemcpyHostToDevice, s));
    }
    *out = r;
    return HEXGEN_OK;
}

KvGeom geom(const hexgen_stage *st, const hexgen_kv_cache *kv) {
    KvGeom g;
    g.d = st->d;
    g.hkv_l = st->hkv_l;
    g.smax = kv->smax;
    g.seq_stride = (int64_t)st->hkv_l * kv->smax * st->d;
    return g;
}

// ---- bf16 prefill flow: five kernels per layer; RoPE / cache append, residual + next-norm operand and SwiGLU
// run in the GEMM epilogues, RMSNorm enters as a per-token scale after the contraction ---------------------
GemmEpi gemm_epi_base(hexgen_stage *st, int mode) {
    GemmEpi e;
    std::memset(&e, 0, sizeof(e));
    e.mode = mode;
    e.norm_dim = st->H;
    e.eps = st->eps;
    return e;
}

void gemm_h16(hexgen_stage *st, const Rows &r, const void *Wp, const h16_t *Xp, int N, int K, const GemmEpi &e,
               int slot, hipStream_t s) {
    st->prof.mark(slot, s);
    HX_K(st->dtype, launch_gemm_mfma, static_cast<const h16_t *>(Wp), Xp, N, K, r.T, e, st->ws.gemm_part, st->ws.gemm_part_floats, s);
    st->prof.mark(slot, s);
}

// QKV projection (+RoPE, cache append) and causal attention; leaves o (fragment tiles) in the workspace
void attn_prefill_h16(hexgen_stage *st, hexgen_kv_cache *kv, int layer, const Rows &r, const float *ssq_in,
                       hipStream_t s) {
    Workspace &w = st->ws;
    const Layer &ly = st->layers[layer];
    const KvGeom kg = geom(st, kv);
    h16_t *kc = static_cast<h16_t *>(kv->k) + (size_t)layer * kv->layer_stride;
    h16_t *vc = static_cast<h16_t *>(kv->v) + (size_t)layer * kv->layer_stride;
    GemmEpi e = gemm_epi_base(st, DEC_QKV);
    e.ssq_in = ssq_in;
    e.hq_l = st->hq_l; e.kg = kg; e.rm = r.rm; e.cos_tab = kv->cos_tab; e.sin_tab = kv->sin_tab;
    e.q = w.q; e.kc = kc; e.vc = vc;
    gemm_h16(st, r, ly.wqkv, w.n, st->nqkv, st->H, e, PROF_QKV, s);
    st->prof.mark(PROF_ATTN, s);
    // one new row per sequence (a decode step of more than 32 sequences): the decode attention kernel, which shares
    // every K / V fragment among the query heads of its kv head, on this path's layouts (row = sequence)
    if (r.max_new == 1 && st->hq_l / st->hkv_l <= 16)
        HX_K(st->dtype, launch_attn_decode_rows, w.q, kc, vc, kg, st->hq_l, w.pos0, r.batch, w.o, s);
    else
        HX_K(st->dtype, launch_attn_prefill, w.q, kc, vc, kg, st->hq_l, w.cu_rows, w.pos0, w.items, r.n_items, w.o, s);
    st->prof.mark(PROF_ATTN, s);
}

hexgen_status_t forward_prefill_h16(hexgen_stage *st, hexgen_kv_cache *kv, const Rows &r, const void *hidden_in,
                                     void *out_partial, void *out_resid, hipStream_t s) {
    Workspace &w = st->ws;
    float *ssq_a = w.ssq_pf, *ssq_f = w.ssq_pf + (size_t)(st->H / GEMM_SSQ_COLS) * r.T;
    HX_K(st->dtype, launch_prefill_prologue, hidden_in, 1, w.h, st->layers[0].g_attn, w.n, ssq_a, r.T, st->H, s);
    for (int l = 0; l < st->L; ++l) {
        const Layer &ly = st->layers[l];
        const bool last = l + 1 == st->L;
        if (st->taps[l]) HX_K(st->dtype, launch_untile_h, w.h, static_cast<float *>(st->taps[l]), r.T, st->H, s);
        attn_prefill_h16(st, kv, l, r, ssq_a, s);
        GemmEpi e = gemm_epi_base(st, DEC_RESID);
        e.h = w.h; e.g_next = ly.g_ffn; e.hg = w.n; e.ssq_out = ssq_f;
        gemm_h16(st, r, ly.wo, w.o, st->H, st->qw, e, PROF_WO, s);
        e = gemm_epi_base(st, DEC_SWIGLU);
        e.ssq_in = ssq_f; e.u = w.u; e.F_l = st->F_l;
        gemm_h16(st, r, ly.w13, w.n, 2 * st->F_l, st->H, e, PROF_W13, s);
        e = gemm_epi_base(st, DEC_RESID);
        e.h = w.h; e.hg = w.n; e.ssq_out = ssq_a;
        e.g_next = last ? nullptr : st->layers[l + 1].g_attn;
        e.last_layer = last ? 1 : 0;
        e.out_partial = static_cast<h16_t *>(out_partial);
        e.out_resid = static_cast<h16_t *>(out_resid);
        gemm_h16(st, r, ly.w2, w.u, st->H, st->F_l, e, PROF_W2, s);
    }
    return HEXGEN_OK;
}

// one sub-layer for the validation surface, prefill kernels; h fp32 in, raw fp32 partial out
void sublayer_prefill_h16(hexgen_stage *st, hexgen_kv_cache *kv, int layer, int which, const Rows &r, const float *h,
                           float *p_out, hipStream_t s) {
    Workspace &w = st->ws;
    const Layer &ly = st->layers[layer];
    float *ssq = w.ssq_pf;
    GemmEpi e = gemm_epi_base(st, DEC_RAW);
    e.raw_out = p_out;
    HX_K(st->dtype, launch_prefill_prologue, h, 0, nullptr, which == 0 ? ly.g_attn : ly.g_ffn, w.n, ssq, r.T, st->H, s);
    if (which == 0) {
        attn_prefill_h16(st, kv, layer, r, ssq, s);
        gemm_h16(st, r, ly.wo, w.o, st->H, st->qw, e, PROF_WO, s);
    } else {
        GemmEpi g = gemm_epi_base(st, DEC_SWIGLU);
        g.ssq_in = ssq; g.u = w.u; g.F_l = st->F_l;
        gemm_h16(st, r, ly.w13, w.n, 2 * st->F_l, st->H, g, PROF_W13, s);
        gemm_h16(st, r, ly.w2, w.u, st->H, st->F_l, e, PROF_W2, s);
    }
}

// ---- bf16 decode flow (T <= 32 rows): five kernels per layer, everything else fused into their tails ----
int g_attn_split_forced = 0;      // measurement and test hook (hexgen_set_attn_split); 0 = choose

int pick_attn_split(const hexgen_stage *st, const hexgen_kv_cache *kv, int batch) {
    if (g_attn_split_forced > 0) return g_attn_split_forced;
    int mx = 0;
    for (int i = 0; i < batch; ++i) mx = std::max(mx, kv->lens[i] + 1);
    const int n_t32 = (mx + 31) / 32;
    // Enough (sequence, kv head) pairs to fill the chip, or a context short enough that one block's eight waves walk it
    // in a few steps: one block per pair.  (Measured on a ragged batch of 32 x 8 pairs, contexts 240..4027: the launch
    // ends 11 us after the same bytes in equal contexts would, but every way of cutting the long contexts -- evenly, or
    // only those above the even share per CU -- costs more than that: a block's fixed part, query load and the merge of
    // its waves, is about 7 us and a CU holds one 8-wave block at a time.)
    // Otherwise every context is split evenly: a block's time falls with the number of splits (one CU's load path
    // delivers about 150 GB/s), while every block adds its own tail (partials written through, the count, the merge);
    // the measured optimum sits near sqrt(4 tiles / pairs).
    const int pairs = batch * st->hkv_l;
    if (pairs >= 32 || n_t32 <= 48) return 1;
    const int s = (int)std::lround(std::sqrt(4.0 * n_t32 / pairs));
    return std::max(2, std::min({s, kStaticAttnSplit, (n_t32 + 7) / 8}));
}

DecodeEpi epi_base(hexgen_stage *st, int mode) {
    DecodeEpi e;
    std::memset(&e, 0, sizeof(e));
    e.mode = mode;
    e.norm_dim = st->H;
    e.ssq_units = st->H / 16;
    e.eps = st->eps;
    return e;
}

void decode_proj(hexgen_stage *st, const Rows &r, const void *Wp, const h16_t *Xa, int N, int K, const DecodeEpi &e,
                 int slot, hipStream_t s) {
    st->prof.mark(slot, s);
    // slot 6: the first kernel of the W1/W3 projection alone (the batched path adds a finishing kernel behind it)
    hipEvent_t mid = nullptr;
    if (slot == PROF_W13 && (st->prof.mask >> PROF_W13_MAIN & 1u)) {
        std::vector<hipEvent_t> &v = st->prof.ev[PROF_W13_MAIN];
        const size_t before = v.size();
        st->prof.mark(PROF_W13_MAIN, s);
        if (v.size() == before + 1 && hipEventCreate(&mid) != hipSuccess) {     // keep start / stop pairs whole
            (void)hipEventDestroy(v.back());
            v.pop_back();
            mid = nullptr;
        }
    }
    HX_K(st->dtype, launch_decode_proj, static_cast<const h16_t *>(Wp), Xa, N, K, r.T, e, st->cur->dec_part, st->cur->dec_part_floats, s, mid);
    if (mid) st->prof.ev[PROF_W13_MAIN].push_back(mid);
    st->prof.mark(slot, s);
}

// QKV (+RoPE, cache append) and attention; leaves o (hi/lo) in the workspace
void attn_decode_h16(hexgen_stage *st, hexgen_kv_cache *kv, int layer, const Rows &r, const float *ssq_in,
                      hipStream_t s) {
    Workspace &w = *st->cur;
    const Layer &ly = st->layers[layer];
    const KvGeom kg = geom(st, kv);
    h16_t *kc = static_cast<h16_t *>(kv->k) + (size_t)layer * kv->layer_stride;
    h16_t *vc = static_cast<h16_t *>(kv->v) + (size_t)layer * kv->layer_stride;
    DecodeEpi e = epi_base(st, DEC_QKV);
    e.ssq_in = ssq_in;
    e.hq_l = st->hq_l; e.kg = kg; e.row_pos = w.row_pos; e.cos_tab = kv->cos_tab; e.sin_tab = kv->sin_tab;
    e.q_hi = w.q; e.q_lo = w.q_lo; e.kc = kc; e.vc = vc;
    // a QKV projection with a split contraction leaves its finishing pass (sum of the partials, 1/rms, rotary
    // embedding, cache append) to the attention kernel, whose blocks own whole heads: one launch less per layer
    QkvTail tail{};
    st->prof.mark(PROF_QKV, s);
    HX_K(st->dtype, launch_decode_qkv, static_cast<const h16_t *>(ly.wqkv), w.xa_n, st->nqkv, st->H, r.T, e, st->cur->dec_part,
         st->cur->dec_part_floats, &tail, s);
    st->prof.mark(PROF_QKV, s);
    st->prof.mark(PROF_ATTN, s);
    HX_K(st->dtype, launch_attn_decode, w.q, w.q_lo, kc, vc, kg, st->hq_l, w.row_pos, r.batch, pick_attn_split(st, kv, r.batch), w.att_o,
                       w.att_ml, w.att_arrived, w.xa_o, tail, s);
    st->prof.mark(PROF_ATTN, s);
}

hexgen_status_t forward_decode_h16(hexgen_stage *st, hexgen_kv_cache *kv, const Rows &r, const void *hidden_in,
                                    void *out_partial, void *out_resid, hipStream_t s) {
    Workspace &w = *st->cur;
    float *ssq_a = w.ssq, *ssq_f = w.ssq + (size_t)(st->H / 16) * DEC_SSQ_STRIDE;
    HX_K(st->dtype, launch_decode_prologue, hidden_in, nullptr, 1, w.h, st->layers[0].g_attn, w.xa_n, ssq_a, r.T, st->H, kv->d_lens,
                           w.row_pos, 1, s);
    for (int l = 0; l < st->L; ++l) {
        const Layer &ly = st->layers[l];
        const bool last = l + 1 == st->L;
        if (st->taps[l])
            HX_HIP(hipMemcpyAsync(st->taps[l], w.h, sizeof(float) * (size_t)r.T * st->H, hipMemcpyDeviceToDevice, s));
        attn_decode_h16(st, kv, l, r, ssq_a, s);
        DecodeEpi e = epi_base(st, DEC_RESID);
        e.h = w.h; e.g_next = ly.g_ffn; e.hg = w.xa_n; e.ssq_out = ssq_f;
        decode_proj(st, r, ly.wo, w.xa_o, st->H, st->qw, e, PROF_WO, s);
        e = epi_base(st, DEC_SWIGLU);
        e.ssq_in = ssq_f; e.u = w.xa_u; e.F_l = st->F_l;
        decode_proj(st, r, ly.w13, w.xa_n, 2 * st->F_l, st->H, e, PROF_W13, s);
        e = epi_base(st, DEC_RESID);
        e.h = w.h; e.hg = w.xa_n; e.ssq_out = ssq_a;
        e.g_next = last ? nullptr : st->layers[l + 1].g_attn;
        e.last_layer = last ? 1 : 0;
        e.out_partial = static_cast<h16_t *>(out_partial);
        e.out_resid = static_cast<h16_t *>(out_resid);
        decode_proj(st, r, ly.w2, w.xa_u, st->H, st->F_l, e, PROF_W2, s);
    }
    return HEXGEN_OK;
}

// one sub-layer for the validation surface, decode kernels; h fp32 in, raw fp32 partial out
void sublayer_decode_h16(hexgen_stage *st, hexgen_kv_cache *kv, int layer, int which, const Rows &r, const float *h,
                          float *p_out, hipStream_t s) {
    Workspace &w = st->ws;
    const Layer &ly = st->layers[layer];
    float *ssq = w.ssq;
    DecodeEpi e = epi_base(st, DEC_RAW);
    e.raw_out = p_out;
    if (which == 0) {
        HX_K(st->dtype, launch_decode_prologue, h, nullptr, 0, nullptr, ly.g_attn, w.xa_n, ssq, r.T, st->H, kv->d_lens, w.row_pos, 0, s);
        attn_decode_h16(st, kv, layer, r, ssq, s);
        decode_proj(st, r, ly.wo, w.xa_o, st->H, st->qw, e, PROF_WO, s);
    } else {
        HX_K(st->dtype, launch_decode_prologue, h, nullptr, 0, nullptr, ly.g_ffn, w.xa_n, ssq, r.T, st->H, nullptr, nullptr, 0, s);
        DecodeEpi g = epi_base(st, DEC_SWIGLU);
        g.ssq_in = ssq; g.u = w.xa_u; g.F_l = st->F_l;
        decode_proj(st, r, ly.w13, w.xa_n, 2 * st->F_l, st->H, g, PROF_W13, s);
        decode_proj(st, r, ly.w2, w.xa_u, st->H, st->F_l, e, PROF_W2, s);
    }
}

hexgen_status_t forward_h16(hexgen_stage *st, hexgen_kv_cache *kv, const Rows &r, const void *hidden_in,
                             void *out_partial, void *out_resid, hipStream_t s) {
    if (r.decode) return forward_decode_h16(st, kv, r, hidden_in, out_partial, out_resid, s);
    return forward_prefill_h16(st, kv, r, hidden_in, out_partial, out_resid, s);
}

// ---- fp32 path -------------------------------------------------------------------------------
void attn_f32(hexgen_stage *st, hexgen_kv_cache *kv, int layer, const Rows &r, const float *h, float *p_out,
              hipStream_t s) {
    Workspace &w = st->ws;
    const Layer &ly = st->layers[layer];
    float *kc = static_cast<float *>(kv->k) + (size_t)layer * kv->layer_stride;
    float *vc = static_cast<float *>(kv->v) + (size_t)layer * kv->layer_stride;
    f32_launch_rmsnorm(h, ly.g_attn, w.n32, r.T, st->H, st->eps, s);
    f32_launch_gemm(w.n32, static_cast<const float *>(ly.wqkv), w.part, r.T, st->H, st->nqkv, s);
    f32_launch_rope_append(w.part, r.T, st->hq_l, st->hkv_l, st->d, kv->smax, r.rm, kv->cos_tab, kv->sin_tab, w.q32, kc,
                           vc, s);
    f32_launch_attn(w.q32, kc, vc, r.T, st->hq_l, st->hkv_l, st->d, kv->smax, r.rm, w.o32, s);
    f32_launch_gemm(w.o32, static_cast<const float *>(ly.wo), p_out, r.T, st->qw, st->H, s);
}
void ffn_f32(hexgen_stage *st, int layer, const Rows &r, const float *h, float *p_out, hipStream_t s) {
    Workspace &w = st->ws;
    const Layer &ly = st->layers[layer];
    f32_launch_rmsnorm(h, ly.g_ffn, w.n32, r.T, st->H, st->eps, s);
    f32_launch_gemm(w.n32, static_cast<const float *>(ly.w13), w.part, r.T, st->H, 2 * st->F_l, s);
    f32_launch_swiglu(w.part, w.u32, r.T, st->F_l, s);
    f32_launch_gemm(w.u32, static_cast<const float *>(ly.w2), p_out, r.T, st->F_l, st->H, s);
}
hexgen_status_t forward_f32(hexgen_stage *st, hexgen_kv_cache *kv, const Rows &r, const void *hidden_in,
                            void *out_partial, void *out_resid, hipStream_t s) {
    Workspace &w = st->ws;
    const size_t bytes = sizeof(float) * (size_t)r.T * st->H;
    HX_HIP(hipMemcpyAsync(w.h, hidden_in, bytes, hipMemcpyDeviceToDevice, s));
    for (int l = 0; l < st->L; ++l) {
        if (st->taps[l]) HX_HIP(hipMemcpyAsync(st->taps[l], w.h, bytes, hipMemcpyDeviceToDevice, s));
        attn_f32(st, kv, l, r, w.h, w.p32, s);
        launch_accumulate_f32(w.h, w.p32, (int64_t)r.T * st->H, s);
        ffn_f32(st, l, r, w.h, w.p32, s);
        if (l + 1 < st->L) {
            launch_accumulate_f32(w.h, w.p32, (int64_t)r.T * st->H, s);
        } else {
            HX_HIP(hipMemcpyAsync(out_partial, w.p32, bytes, hipMemcpyDeviceToDevice, s));
            if (out_resid) HX_HIP(hipMemcpyAsync(out_resid, w.h, bytes, hipMemcpyDeviceToDevice, s));
        }
    }
    return HEXGEN_OK;
}

hexgen_status_t check_loaded(const hexgen_stage *st) {
    for (const Layer &l : st->layers)
        if (!l.loaded) return HEXGEN_ERR_STATE;
    return HEXGEN_OK;
}

// the cache's rotation tables were built for the theta the stage had when the cache was created
hexgen_status_t check_rope(const hexgen_stage *st, const hexgen_kv_cache *kv) {
    return kv->rope_theta_built == st->theta ? HEXGEN_OK : HEXGEN_ERR_STATE;
}

hexgen_status_t upload_lens(hexgen_kv_cache *kv) {
    HX_HIP(hipMemcpy(kv->d_lens, kv->lens.data(), sizeof(int32_t) * kv->max_batch, hipMemcpyHostToDevice));
    return HEXGEN_OK;
}

void free_layer(Layer &l) {
    void *ptrs[] = {l.g_attn, l.g_ffn, l.wqkv, l.wo, l.w13, l.w2};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    l = Layer();
}


// ---- the allocation-free decode step: its whole workspace lives in one file-scope device array ------------------
constexpr size_t kStaticScratchBytes = (size_t)HEXGEN_STATIC_SCRATCH_BYTES;
constexpr int kStaticMaxDevices = 64;

}  // namespace

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.  In
// host code the name below is only a handle for hipGetSymbolAddress: the device address is looked up once per
// device (static_scratch_ptr) and that pointer is what kernels and fills receive.
static __device__ __align__(256) unsigned char hexgen_static_scratch[kStaticScratchBytes];

namespace {

void *g_static_scratch_ptr[kStaticMaxDevices];          // per device, nullptr until looked up

hexgen_status_t static_scratch_ptr(unsigned char **out) {
    int dev = -1;
    HX_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticMaxDevices) return HEXGEN_ERR_DEVICE;
    if (!g_static_scratch_ptr[dev]) {
        void *p = nullptr;
        HX_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(hexgen_static_scratch)));
        if (!p) return HEXGEN_ERR_DEVICE;
        g_static_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char *>(g_static_scratch_ptr[dev]);
    return HEXGEN_OK;
}

// Lays the buffers of one decode call of `rows` rows out behind `base` (256-byte aligned pieces) and returns the bytes
// used; with base == nullptr only the size is computed.  Same buffers, sizes per row and roles as ensure_workspace's
// decode part; the attention partials are sized for the 8 splits the split rule allows.
size_t carve_decode_workspace(const hexgen_stage *st, int rows, unsigned char *base, Workspace *w) {
    size_t off = 0;
    auto take = [&](size_t bytes) -> void * {
        off = (off + 255) / 256 * 256;
        void *p = base ? base + off : nullptr;
        off += bytes;
        return p;
    };
    const size_t T = (size_t)rows;
    const size_t nmax = (size_t)std::max(std::max(st->nqkv, st->H), 2 * st->F_l);
    Workspace v;
    v.cap_rows = rows;
    v.h = static_cast<float *>(take(T * st->H * sizeof(float)));
    v.xa_n = static_cast<h16_t *>(take(2 * T * st->H * sizeof(h16_t)));
    v.xa_o = static_cast<h16_t *>(take(2 * T * st->qw * sizeof(h16_t)));
    v.xa_u = static_cast<h16_t *>(take(2 * T * st->F_l * sizeof(h16_t)));
    v.q = static_cast<h16_t *>(take(T * st->qw * sizeof(h16_t)));
    v.q_lo = static_cast<h16_t *>(take(T * st->qw * sizeof(h16_t)));
    if (rows > 2) {
        v.dec_part_floats = T * ((size_t)512 * 128 + 2 * nmax);
        v.dec_part = static_cast<float *>(take(v.dec_part_floats * sizeof(float)));
    }
    v.att_o = static_cast<float *>(take(T * st->hq_l * kStaticAttnSplit * st->d * sizeof(float)));
    v.att_ml = static_cast<float *>(take(T * st->hq_l * kStaticAttnSplit * 2 * sizeof(float)));
    v.att_arrived = static_cast<unsigned int *>(take(T * st->hkv_l * sizeof(unsigned int)));
    v.ssq = static_cast<float *>(take(2 * (size_t)(st->H / 16) * DEC_SSQ_STRIDE * sizeof(float)));
    v.row_pos = static_cast<int32_t *>(take(T * sizeof(int32_t)));
    if (w) *w = v;
    return off;
}

}  // namespace

// =================================================================================================
extern "C" {

const char *hexgen_status_string(hexgen_status_t s) {
    switch (s) {
        case HEXGEN_OK: return "ok";
        case HEXGEN_ERR_INVALID_ARG: return "invalid argument";
        case HEXGEN_ERR_SHAPE: return "shape not supported / sharding does not divide";
        case HEXGEN_ERR_STATE: return "call not valid in the current state";
        case HEXGEN_ERR_CAPACITY: return "capacity exceeded";
        case HEXGEN_ERR_OOM: return "out of memory";
        case HEXGEN_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

hexgen_status_t hexgen_stage_create(int hidden, int n_heads, int n_kv_heads, int ffn, int n_layers, int tp_degree,
                                    int tp_rank, hexgen_dtype_t dtype, hexgen_stage_t **out) {
    if (!out) return HEXGEN_ERR_INVALID_ARG;
    if (hidden <= 0 || n_heads <= 0 || n_kv_heads <= 0 || ffn <= 0 || n_layers <= 0 || tp_degree <= 0)
        return HEXGEN_ERR_INVALID_ARG;
    if (!known_dtype(dtype)) return HEXGEN_ERR_INVALID_ARG;
    if (tp_rank < 0 || tp_rank >= tp_degree) return HEXGEN_ERR_SHAPE;
    if (hidden % n_heads || n_heads % n_kv_heads || n_heads % tp_degree || n_kv_heads % tp_degree ||
        ffn % tp_degree)
        return HEXGEN_ERR_SHAPE;
    const int d = hidden / n_heads;
    if (d != 64 && d != 128) return HEXGEN_ERR_SHAPE;
    const int hq_l = n_heads / tp_degree, hkv_l = n_kv_heads / tp_degree, F_l = ffn / tp_degree;
    if (hq_l / hkv_l > 16) return HEXGEN_ERR_SHAPE;          // one MFMA column block per query group
    if (is_h16(dtype) && (hidden % 128 || (hq_l * d) % 32 || F_l % 32)) return HEXGEN_ERR_SHAPE;
    if (hidden % 8) return HEXGEN_ERR_SHAPE;
    hexgen_stage *st = new (std::nothrow) hexgen_stage();
    if (!st) return HEXGEN_ERR_OOM;
    st->H = hidden; st->hq = n_heads; st->hkv = n_kv_heads; st->F = ffn; st->L = n_layers;
    st->t = tp_degree; st->r = tp_rank; st->d = d; st->hq_l = hq_l; st->hkv_l = hkv_l; st->F_l = F_l;
    st->qw = hq_l * d;
    st->nqkv = (hq_l + 2 * hkv_l) * d;
    st->dtype = dtype;
    st->cur = &st->ws;
    try {       // no exception may cross the C boundary
        st->layers.resize(n_layers);
        st->taps.assign(n_layers, nullptr);
    } catch (...) {
        delete st;
        return HEXGEN_ERR_OOM;
    }
    *out = st;
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stage_set_params(hexgen_stage_t *st, float rms_eps, float rope_theta) {
    if (!st || !(rms_eps >= 0.f) || !(rope_theta > 0.f)) return HEXGEN_ERR_INVALID_ARG;
    st->eps = rms_eps;
    st->theta = rope_theta;
    return HEXGEN_OK;
}

void hexgen_stage_destroy(hexgen_stage_t *st) {
    if (!st) return;
    (void)hipDeviceSynchronize();
    for (Layer &l : st->layers) free_layer(l);
    free_ws(st->ws);
    st->prof.clear();
    delete st;
}

int64_t hexgen_stage_weight_bytes(const hexgen_stage_t *st) { return st ? st->weight_bytes : 0; }

hexgen_status_t hexgen_stage_load_layer(hexgen_stage_t *st, int layer, const void *g_attn, const void *wq,
                                        const void *wk, const void *wv, const void *wo, const void *g_ffn,
                                        const void *w1, const void *w3, const void *w2) {
    if (!st || !g_attn || !wq || !wk || !wv || !wo || !g_ffn || !w1 || !w3 || !w2) return HEXGEN_ERR_INVALID_ARG;
    if (layer < 0 || layer >= st->L) return HEXGEN_ERR_INVALID_ARG;
    HX_HIP(hipDeviceSynchronize());
    Layer &ly = st->layers[layer];
    if (ly.loaded) st->weight_bytes -= (int64_t)esize(st->dtype) * ((int64_t)st->H * st->nqkv + (int64_t)st->qw * st->H +
                                                                   3LL * st->H * st->F_l);
    free_layer(ly);
    const int H = st->H, d = st->d, r = st->r;
    const size_t es = esize(st->dtype);
    const int qcols = st->hq * d, kcols = st->hkv * d;     // global widths
    const int q0 = r * st->qw, k0 = r * st->hkv_l * d, f0 = r * st->F_l, kw = st->hkv_l * d;

    // gains -> fp32 on device
    HX_TRY(dmalloc(&ly.g_attn, (size_t)H));
    HX_TRY(dmalloc(&ly.g_ffn, (size_t)H));
    if (st->dtype == HEXGEN_F32) {
        HX_HIP(hipMemcpy(ly.g_attn, g_attn, sizeof(float) * H, hipMemcpyDefault));
        HX_HIP(hipMemcpy(ly.g_ffn, g_ffn, sizeof(float) * H, hipMemcpyDefault));
    } else {
        h16_t *tmp = nullptr;
        HX_TRY(dmalloc(&tmp, (size_t)2 * H));
        hipError_t e1 = hipMemcpy(tmp, g_attn, sizeof(h16_t) * H, hipMemcpyDefault);
        hipError_t e2 = hipMemcpy(tmp + H, g_ffn, sizeof(h16_t) * H, hipMemcpyDefault);
        if (e1 == hipSuccess && e2 == hipSuccess) {
            HX_K(st->dtype, launch_cvt_h16_to_f32, tmp, ly.g_attn, H, nullptr);
            HX_K(st->dtype, launch_cvt_h16_to_f32, tmp + H, ly.g_ffn, H, nullptr);
            e1 = hipDeviceSynchronize();
        }
        (void)hipFree(tmp);
        HX_HIP(e1);
        HX_HIP(e2);
    }

    const size_t n_qkv = (size_t)H * st->nqkv, n_wo = (size_t)st->qw * H, n_13 = (size_t)H * 2 * st->F_l,
                 n_w2 = (size_t)st->F_l * H;
    HX_HIP(hipMalloc(&ly.wqkv, n_qkv * es));
    HX_HIP(hipMalloc(&ly.wo, n_wo * es));
    HX_HIP(hipMalloc(&ly.w13, n_13 * es));
    HX_HIP(hipMalloc(&ly.w2, n_w2 * es));

    auto cbytes = [&](int cols) { return (size_t)cols * es; };
    auto src_at = [&](const void *base, size_t row, size_t col, size_t ld) {
        return static_cast<const char *>(base) + (row * ld + col) * es;
    };
    if (st->dtype == HEXGEN_F32) {
        // plain layouts: wqkv [H][q | k | v], w13 [H][w1 | w3]; row shards are contiguous
        char *qkv = static_cast<char *>(ly.wqkv);
        HX_HIP(hipMemcpy2D(qkv, cbytes(st->nqkv), src_at(wq, 0, q0, qcols), cbytes(qcols), cbytes(st->qw), H,
                           hipMemcpyDefault));
        HX_HIP(hipMemcpy2D(qkv + cbytes(st->qw), cbytes(st->nqkv), src_at(wk, 0, k0, kcols), cbytes(kcols), cbytes(kw),
                           H, hipMemcpyDefault));
        HX_HIP(hipMemcpy2D(qkv + cbytes(st->qw + kw), cbytes(st->nqkv), src_at(wv, 0, k0, kcols), cbytes(kcols),
                           cbytes(kw), H, hipMemcpyDefault));
        char *w13 = static_cast<char *>(ly.w13);
        HX_HIP(hipMemcpy2D(w13, cbytes(2 * st->F_l), src_at(w1, 0, f0, st->F), cbytes(st->F), cbytes(st->F_l), H,
                           hipMemcpyDefault));
        HX_HIP(hipMemcpy2D(w13 + cbytes(st->F_l), cbytes(2 * st->F_l), src_at(w3, 0, f0, st->F), cbytes(st->F),
                           cbytes(st->F_l), H, hipMemcpyDefault));
        HX_HIP(hipMemcpy(ly.wo, src_at(wo, q0, 0, H), n_wo * es, hipMemcpyDefault));
        HX_HIP(hipMemcpy(ly.w2, src_at(w2, f0, 0, H), n_w2 * es, hipMemcpyDefault));
    } else {
        // stage each shard in a dense device buffer, then repack it into MFMA fragment order
        const size_t tmp_elems = std::max(std::max((size_t)H * st->qw, (size_t)H * st->F_l), n_wo);
        h16_t *tmp = nullptr;
        HX_TRY(dmalloc(&tmp, tmp_elems));
        hexgen_status_t rc = HEXGEN_OK;
        auto col_shard = [&](const void *src, int c0, int gcols, int cols, void *dst, int tile0, int stride, int dst_tiles,
                             int rope_d) {
            if (rc != HEXGEN_OK) return;
            hipError_t e = hipMemcpy2D(tmp, cbytes(cols), src_at(src, 0, c0, gcols), cbytes(gcols), cbytes(cols), H,
                                       hipMemcpyDefault);
            if (e != hipSuccess) { rc = HEXGEN_ERR_DEVICE; return; }
            launch_pack_weight(tmp, cols, 0, 0, H, cols, static_cast<h16_t *>(dst), tile0, stride, dst_tiles, rope_d, nullptr);
            if (hipDeviceSynchronize() != hipSuccess) rc = HEXGEN_ERR_DEVICE;
        };
        auto row_shard = [&](const void *src, int r0, int rows, void *dst) {
            if (rc != HEXGEN_OK) return;
            hipError_t e = hipMemcpy(tmp, src_at(src, r0, 0, H), (size_t)rows * H * es, hipMemcpyDefault);
            if (e != hipSuccess) { rc = HEXGEN_ERR_DEVICE; return; }
            launch_pack_weight(tmp, H, 0, 0, rows, H, static_cast<h16_t *>(dst), 0, 1, H / 16, 0, nullptr);
            if (hipDeviceSynchronize() != hipSuccess) rc = HEXGEN_ERR_DEVICE;
        };
        col_shard(wq, q0, qcols, st->qw, ly.wqkv, 0, 1, st->nqkv / 16, d);        // q, k, v tiles hold rotary pairs
        col_shard(wk, k0, kcols, kw, ly.wqkv, st->qw / 16, 1, st->nqkv / 16, d);
        col_shard(wv, k0, kcols, kw, ly.wqkv, (st->qw + kw) / 16, 1, st->nqkv / 16, d);
        col_shard(w1, f0, st->F, st->F_l, ly.w13, 0, 2, st->F_l / 8, 0);  // gate tiles at even positions
        col_shard(w3, f0, st->F, st->F_l, ly.w13, 1, 2, st->F_l / 8, 0);  // up tiles at odd positions
        row_shard(wo, q0, st->qw, ly.wo);
        row_shard(w2, f0, st->F_l, ly.w2);
        (void)hipFree(tmp);
        if (rc != HEXGEN_OK) { (void)hipGetLastError(); free_layer(ly); return rc; }
    }
    ly.loaded = true;
    st->weight_bytes += (int64_t)es * (int64_t)(n_qkv + n_wo + n_13 + n_w2);
    return HEXGEN_OK;
}

// ---- KV cache ------------------------------------------------------------------------------------
hexgen_status_t hexgen_kv_cache_create(hexgen_stage_t *st, int max_batch, int max_seq, hexgen_kv_cache_t **out) {
    if (!st || !out || max_batch <= 0 || max_seq <= 0) return HEXGEN_ERR_INVALID_ARG;
    if (st->dtype == HEXGEN_F32 && max_seq > 8192) return HEXGEN_ERR_CAPACITY;   // fp32 attention keeps scores in LDS
    hexgen_kv_cache *kv = new (std::nothrow) hexgen_kv_cache();
    if (!kv) return HEXGEN_ERR_OOM;
    kv->st = st;
    kv->max_batch = max_batch;
    kv->max_seq = max_seq;
    kv->smax = round_up(max_seq, 32);
    kv->layer_stride = (int64_t)max_batch * st->hkv_l * kv->smax * st->d;
    kv->lens.assign(max_batch, 0);
    const size_t bytes = (size_t)st->L * kv->layer_stride * esize(st->dtype);
    const int half = st->d / 2;
    std::vector<float> cs((size_t)kv->smax * half), sn((size_t)kv->smax * half);
    for (int p = 0; p < kv->smax; ++p)
        for (int i = 0; i < half; ++i) {
            const double ang = (double)p * std::pow((double)st->theta, -2.0 * i / st->d);
            cs[(size_t)p * half + i] = (float)std::cos(ang);
            sn[(size_t)p * half + i] = (float)std::sin(ang);
        }
    hipError_t e = hipMalloc(&kv->k, bytes);
    if (e == hipSuccess) e = hipMalloc(&kv->v, bytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&kv->cos_tab), cs.size() * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&kv->sin_tab), sn.size() * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&kv->d_lens), sizeof(int32_t) * max_batch);
    if (e == hipSuccess) e = hipMemset(kv->k, 0, bytes);
    if (e == hipSuccess) e = hipMemset(kv->v, 0, bytes);
    if (e == hipSuccess) e = hipMemset(kv->d_lens, 0, sizeof(int32_t) * max_batch);
    if (e == hipSuccess) e = hipMemcpy(kv->cos_tab, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(kv->sin_tab, sn.data(), sn.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipGetLastError();
        hexgen_kv_cache_destroy(kv);
        return e == hipErrorOutOfMemory ? HEXGEN_ERR_OOM : HEXGEN_ERR_DEVICE;
    }
    kv->rope_theta_built = st->theta;
    *out = kv;
    return HEXGEN_OK;
}

void hexgen_kv_cache_destroy(hexgen_kv_cache_t *kv) {
    if (!kv) return;
    (void)hipDeviceSynchronize();
    void *ptrs[] = {kv->k, kv->v, kv->cos_tab, kv->sin_tab, kv->d_lens};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete kv;
}

hexgen_status_t hexgen_kv_cache_reset(hexgen_kv_cache_t *kv) {
    if (!kv) return HEXGEN_ERR_INVALID_ARG;
    HX_HIP(hipDeviceSynchronize());
    std::fill(kv->lens.begin(), kv->lens.end(), 0);
    kv->batch = 0;
    kv->prefilled = false;
    kv->steps = 0;
    return upload_lens(kv);
}

hexgen_status_t hexgen_kv_cache_set_lengths(hexgen_kv_cache_t *kv, const int32_t *lens, int batch) {
    if (!kv || !lens || batch <= 0) return HEXGEN_ERR_INVALID_ARG;
    if (batch > kv->max_batch) return HEXGEN_ERR_CAPACITY;
    for (int i = 0; i < batch; ++i) {
        if (lens[i] < 0) return HEXGEN_ERR_INVALID_ARG;
        if (lens[i] > kv->max_seq) return HEXGEN_ERR_CAPACITY;
    }
    HX_HIP(hipDeviceSynchronize());
    std::fill(kv->lens.begin(), kv->lens.end(), 0);
    for (int i = 0; i < batch; ++i) kv->lens[i] = lens[i];
    kv->batch = batch;
    kv->prefilled = true;
    kv->steps = 0;
    return upload_lens(kv);
}

hexgen_status_t hexgen_kv_cache_get_lengths(hexgen_kv_cache_t *kv, int32_t *lens_out, int batch) {
    if (!kv || !lens_out || batch <= 0 || batch > kv->max_batch) return HEXGEN_ERR_INVALID_ARG;
    for (int i = 0; i < batch; ++i) lens_out[i] = kv->lens[i];
    return HEXGEN_OK;
}

hexgen_status_t hexgen_kv_cache_commit(hexgen_kv_cache_t *kv, const int32_t *seq_lens, int batch) {
    if (!kv || batch <= 0) return HEXGEN_ERR_INVALID_ARG;
    if (batch > kv->max_batch) return HEXGEN_ERR_CAPACITY;
    for (int i = 0; i < batch; ++i) {
        const int n = seq_lens ? seq_lens[i] : 1;
        if (n < 0) return HEXGEN_ERR_INVALID_ARG;
        if ((long)kv->lens[i] + n > kv->max_seq) return HEXGEN_ERR_CAPACITY;
    }
    HX_HIP(hipDeviceSynchronize());
    for (int i = 0; i < batch; ++i) kv->lens[i] += seq_lens ? seq_lens[i] : 1;
    kv->batch = std::max(kv->batch, batch);
    kv->prefilled = true;
    return upload_lens(kv);
}

static hexgen_status_t kv_io(hexgen_kv_cache_t *kv, int layer, int seq, int pos0, int n, float *k, float *v,
                             bool to_cache) {
    if (!kv || !k || !v) return HEXGEN_ERR_INVALID_ARG;
    hexgen_stage *st = kv->st;
    if (layer < 0 || layer >= st->L || seq < 0 || seq >= kv->max_batch || pos0 < 0 || n < 0)
        return HEXGEN_ERR_INVALID_ARG;
    if ((long)pos0 + n > kv->max_seq) return HEXGEN_ERR_CAPACITY;
    if (n == 0) return HEXGEN_OK;
    HX_HIP(hipDeviceSynchronize());
    const size_t cnt = (size_t)n * st->hkv_l * st->d;
    float *dk = nullptr, *dv = nullptr;
    HX_TRY(dmalloc(&dk, cnt));
    hexgen_status_t rc = dmalloc(&dv, cnt);
    if (rc != HEXGEN_OK) { (void)hipFree(dk); return rc; }
    hipError_t e = hipSuccess;
    if (to_cache) {
        e = hipMemcpy(dk, k, cnt * sizeof(float), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(dv, v, cnt * sizeof(float), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) {
        if (is_h16(st->dtype)) {
            h16_t *kc = static_cast<h16_t *>(kv->k) + (size_t)layer * kv->layer_stride;
            h16_t *vc = static_cast<h16_t *>(kv->v) + (size_t)layer * kv->layer_stride;
            if (to_cache) HX_K(st->dtype, launch_kv_scatter, dk, dv, kc, vc, geom(st, kv), seq, pos0, n, nullptr);
            else HX_K(st->dtype, launch_kv_gather, kc, vc, geom(st, kv), seq, pos0, n, dk, dv, nullptr);
        } else {
            float *kc = static_cast<float *>(kv->k) + (size_t)layer * kv->layer_stride;
            float *vc = static_cast<float *>(kv->v) + (size_t)layer * kv->layer_stride;
            f32_launch_kv_copy(kc, vc, dk, dv, st->hkv_l, st->d, kv->smax, seq, pos0, n, to_cache ? 1 : 0, nullptr);
        }
        e = hipDeviceSynchronize();
    }
    if (e == hipSuccess && !to_cache) {
        e = hipMemcpy(k, dk, cnt * sizeof(float), hipMemcpyDeviceToHost);
        if (e == hipSuccess) e = hipMemcpy(v, dv, cnt * sizeof(float), hipMemcpyDeviceToHost);
    }
    (void)hipFree(dk);
    (void)hipFree(dv);
    HX_HIP(e);
    return HEXGEN_OK;
}

hexgen_status_t hexgen_kv_cache_read(hexgen_kv_cache_t *kv, int layer, int seq, int pos0, int n, float *k_out,
                                     float *v_out) {
    return kv_io(kv, layer, seq, pos0, n, k_out, v_out, false);
}
hexgen_status_t hexgen_kv_cache_fill(hexgen_kv_cache_t *kv, int layer, int seq, int n, const float *k,
                                     const float *v) {
    return kv_io(kv, layer, seq, 0, n, const_cast<float *>(k), const_cast<float *>(v), true);
}

// ---- prefill / decode ------------------------------------------------------------------------------
hexgen_status_t hexgen_stage_prefill(hexgen_stage_t *st, hexgen_kv_cache_t *kv, const void *hidden_in,
                                     const int32_t *seq_lens, int batch, void *out_partial, void *out_resid,
                                     void *stream) {
    if (!st || !kv || !hidden_in || !seq_lens || !out_partial || kv->st != st) return HEXGEN_ERR_INVALID_ARG;
    HX_TRY(check_loaded(st));
    if (batch <= 0) return HEXGEN_ERR_INVALID_ARG;
    if (batch > kv->max_batch) return HEXGEN_ERR_CAPACITY;
    for (int i = 0; i < batch; ++i) {
        if (seq_lens[i] < 1) return HEXGEN_ERR_INVALID_ARG;
        if (seq_lens[i] > kv->max_seq) return HEXGEN_ERR_CAPACITY;
    }
    HX_TRY(check_rope(st, kv));
    hipStream_t s = static_cast<hipStream_t>(stream);
    long total = 0;
    for (int i = 0; i < batch; ++i) total += seq_lens[i];
    if (total > 0x3fffffff) return HEXGEN_ERR_CAPACITY;
    HX_TRY(ensure_workspace(st, (int)total, batch));     // every check that can fail comes before the cache is touched
    HX_TRY(hexgen_kv_cache_reset(kv));
    Rows r;
    HX_TRY(setup_rows(st, kv, seq_lens, batch, false, s, &r));      // a prefill always takes the GEMM path
    st->prof.mark(PROF_CALL, s);
    if (is_h16(st->dtype)) HX_TRY(forward_h16(st, kv, r, hidden_in, out_partial, out_resid, s));
    else HX_TRY(forward_f32(st, kv, r, hidden_in, out_partial, out_resid, s));
    st->prof.mark(PROF_CALL, s);
    for (int i = 0; i < batch; ++i) kv->lens[i] = seq_lens[i];
    kv->batch = batch;
    kv->prefilled = true;
    kv->steps = 0;
    // the new lengths reach the device in stream order, behind the kernels of this call
    int32_t *h_len = st->ws.host_stage + 2 * r.T + 2 * batch + 1;
    for (int i = 0; i < batch; ++i) h_len[i] = seq_lens[i];
    HX_HIP(hipMemcpyAsync(kv->d_lens, h_len, sizeof(int32_t) * batch, hipMemcpyHostToDevice, s));
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stage_decode(hexgen_stage_t *st, hexgen_kv_cache_t *kv, int step, const void *hidden_in,
                                    void *out_partial, void *out_resid, void *stream) {
    if (!st || !kv || !hidden_in || !out_partial || kv->st != st) return HEXGEN_ERR_INVALID_ARG;
    HX_TRY(check_loaded(st));
    if (!kv->prefilled || kv->batch <= 0 || step != kv->steps) return HEXGEN_ERR_STATE;
    HX_TRY(check_rope(st, kv));
    hipStream_t s = static_cast<hipStream_t>(stream);
    Rows r;
    HX_TRY(setup_rows(st, kv, nullptr, kv->batch, true, s, &r));
    st->prof.mark(PROF_CALL, s);
    if (is_h16(st->dtype)) HX_TRY(forward_h16(st, kv, r, hidden_in, out_partial, out_resid, s));
    else HX_TRY(forward_f32(st, kv, r, hidden_in, out_partial, out_resid, s));
    if (r.decode && is_h16(st->dtype)) st->last_decode_rows = r.T;
    if (!r.decode || !is_h16(st->dtype)) launch_advance_lens(kv->d_lens, kv->batch, s);   // else: the prologue did
    st->prof.mark(PROF_CALL, s);
    for (int i = 0; i < kv->batch; ++i) kv->lens[i] += 1;
    kv->steps += 1;
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stage_decode_static(hexgen_stage_t *st, hexgen_kv_cache_t *kv, int step, const void *hidden_in,
                                           void *out_partial, void *out_resid, void *stream) {
    if (!st || !kv || !hidden_in || !out_partial || kv->st != st) return HEXGEN_ERR_INVALID_ARG;
    HX_TRY(check_loaded(st));
    if (!is_h16(st->dtype)) return HEXGEN_ERR_SHAPE;
    if (!kv->prefilled || kv->batch <= 0 || step != kv->steps) return HEXGEN_ERR_STATE;
    HX_TRY(check_rope(st, kv));
    const int batch = kv->batch;
    if (batch > kDecodeMaxRows) return HEXGEN_ERR_CAPACITY;
    for (int i = 0; i < batch; ++i)
        if ((long)kv->lens[i] + 1 > kv->max_seq) return HEXGEN_ERR_CAPACITY;
    if (carve_decode_workspace(st, batch, nullptr, nullptr) > kStaticScratchBytes) return HEXGEN_ERR_CAPACITY;
    unsigned char *base = nullptr;
    HX_TRY(static_scratch_ptr(&base));
    hipStream_t s = static_cast<hipStream_t>(stream);
    Workspace view;
    (void)carve_decode_workspace(st, batch, base, &view);
    // what must start at zero: the arrival counters of the split attention and the sums of squares (a fill kernel,
    // not a memset node, so that the call can be captured into a graph)
    launch_fill_zero(view.att_arrived, (size_t)batch * st->hkv_l * sizeof(unsigned int), s);
    launch_fill_zero(view.ssq, 2 * (size_t)(st->H / 16) * DEC_SSQ_STRIDE * sizeof(float), s);
    Rows r;
    r.T = batch;
    r.batch = batch;
    r.max_new = 1;
    r.decode = true;
    r.rm.row_seq = nullptr;        // the bf16 decode kernels take positions only (published by the prologue)
    r.rm.row_pos = view.row_pos;
    const unsigned saved_mask = st->prof.mask;
    st->prof.mask = 0;             // the timing slots create events: not in a call that allocates nothing
    st->cur = &view;
    const hexgen_status_t rc = forward_decode_h16(st, kv, r, hidden_in, out_partial, out_resid, s);
    st->cur = &st->ws;
    st->prof.mask = saved_mask;
    HX_TRY(rc);
    HX_HIP(hipGetLastError());
    for (int i = 0; i < batch; ++i) kv->lens[i] += 1;
    kv->steps += 1;
    return HEXGEN_OK;
}

int64_t hexgen_stage_decode_static_bytes(const hexgen_stage_t *st, int batch) {
    if (!st || batch <= 0 || !is_h16(st->dtype)) return -1;
    return (int64_t)carve_decode_workspace(st, batch, nullptr, nullptr);
}

// ---- validation surface ----------------------------------------------------------------------------
hexgen_status_t hexgen_stage_run_sublayer(hexgen_stage_t *st, hexgen_kv_cache_t *kv, int layer, int which,
                                          const void *h_in, const int32_t *seq_lens, int batch, void *partial_out,
                                          void *stream) {
    if (!st || !kv || !h_in || !partial_out || kv->st != st) return HEXGEN_ERR_INVALID_ARG;
    if (layer < 0 || layer >= st->L || (which != 0 && which != 1)) return HEXGEN_ERR_INVALID_ARG;
    if (!st->layers[layer].loaded) return HEXGEN_ERR_STATE;
    HX_TRY(check_rope(st, kv));
    hipStream_t s = static_cast<hipStream_t>(stream);
    Rows r;
    HX_TRY(setup_rows(st, kv, seq_lens, batch, true, s, &r));
    const float *h = static_cast<const float *>(h_in);
    float *p = static_cast<float *>(partial_out);
    if (is_h16(st->dtype)) {
        if (r.decode) {
            sublayer_decode_h16(st, kv, layer, which, r, h, p, s);
        } else {
            sublayer_prefill_h16(st, kv, layer, which, r, h, p, s);
        }
    } else {
        if (which == 0) attn_f32(st, kv, layer, r, h, p, s);
        else ffn_f32(st, layer, r, h, p, s);
    }
    return HEXGEN_OK;
}

hexgen_status_t hexgen_accumulate_f32(void *dst, const void *src, int64_t n, void *stream) {
    if (!dst || !src || n < 0) return HEXGEN_ERR_INVALID_ARG;
    launch_accumulate_f32(static_cast<float *>(dst), static_cast<const float *>(src), n, static_cast<hipStream_t>(stream));
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stage_profile_enable(hexgen_stage_t *st, int slot_mask) {
    if (!st || slot_mask < 0 || slot_mask >= (1 << PROF_SLOTS)) return HEXGEN_ERR_INVALID_ARG;
    HX_HIP(hipDeviceSynchronize());
    st->prof.clear();
    st->prof.mask = (unsigned)slot_mask;
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stage_profile_read(hexgen_stage_t *st, int slot, double *total_ms, int64_t *count) {
    if (!st || !total_ms || !count || slot < 0 || slot >= PROF_SLOTS) return HEXGEN_ERR_INVALID_ARG;
    HX_HIP(hipDeviceSynchronize());
    const std::vector<hipEvent_t> &v = st->prof.ev[slot];
    double tot = 0.0;
    int64_t n = 0;
    for (size_t i = 0; i + 1 < v.size(); i += 2) {
        float ms = 0.f;
        HX_HIP(hipEventElapsedTime(&ms, v[i], v[i + 1]));
        tot += ms;
        ++n;
    }
    *total_ms = tot;
    *count = n;
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stage_time_w13_decode(hexgen_stage_t *st, int reps, double *total_ms, int64_t *launches,
                                             void *stream) {
    if (!st || !total_ms || !launches || reps <= 0) return HEXGEN_ERR_INVALID_ARG;
    HX_TRY(check_loaded(st));
    if (!is_h16(st->dtype) || st->last_decode_rows <= 0) return HEXGEN_ERR_STATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Workspace &w = st->ws;
    Rows r;
    r.T = st->last_decode_rows;
    r.batch = r.T;
    r.decode = true;
    hipEvent_t e0, e1;
    HX_HIP(hipEventCreate(&e0));
    HX_HIP(hipEventCreate(&e1));
    const unsigned saved = st->prof.mask;
    st->prof.mask = 0;
    DecodeEpi e = epi_base(st, DEC_SWIGLU);
    e.ssq_in = w.ssq + (size_t)(st->H / 16) * DEC_SSQ_STRIDE;
    e.u = w.xa_u;
    e.F_l = st->F_l;
    HX_HIP(hipEventRecord(e0, s));
    for (int i = 0; i < reps; ++i)
        for (int l = 0; l < st->L; ++l) decode_proj(st, r, st->layers[l].w13, w.xa_n, 2 * st->F_l, st->H, e, PROF_W13, s);
    HX_HIP(hipEventRecord(e1, s));
    HX_HIP(hipEventSynchronize(e1));
    st->prof.mask = saved;
    float ms = 0.f;
    HX_HIP(hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *total_ms = ms;
    *launches = (int64_t)reps * st->L;
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stream_copy(void *dst, const void *src, int64_t bytes, int blocks, void *stream) {
    if (!dst || !src || bytes < 0 || bytes % 16 || blocks <= 0) return HEXGEN_ERR_INVALID_ARG;
    launch_stream_copy(src, dst, bytes, blocks, static_cast<hipStream_t>(stream));
    return HEXGEN_OK;
}

hexgen_status_t hexgen_stream_read(const void *src, void *sink, int64_t bytes, int blocks, void *stream) {
    if (!sink || !src || bytes < 0 || bytes % 16 || blocks <= 0) return HEXGEN_ERR_INVALID_ARG;
    launch_stream_read(src, static_cast<float *>(sink), bytes, blocks, static_cast<hipStream_t>(stream));
    return HEXGEN_OK;
}

hexgen_status_t hexgen_mfma_probe(int variant, void *sink, int iters, int blocks, void *stream) {
    if (!sink || variant < 0 || variant > 11 || iters <= 0 || blocks <= 0) return HEXGEN_ERR_INVALID_ARG;
    launch_mfma_probe(variant, static_cast<float *>(sink), iters, blocks, static_cast<hipStream_t>(stream));
    return HEXGEN_OK;
}

// ---- the model's ends next to the stage: embedding gather, final norm + vocabulary-parallel LM head + argmax ----
struct hexgen_head {
    int H = 0, V = 0, t = 1, r = 0, Vl = 0, Vpad = 0;     // Vl = V / t columns of this rank, padded to 16 for the tiles
    hexgen_dtype_t dtype = HEXGEN_BF16;
    float eps = 1e-5f;
    bool loaded = false;
    void *w = nullptr;            // bf16: fragment tiles, k-tile-major [H/32][Vpad/16][64][8]; f32: [H][Vl]
    float *g = nullptr;           // final norm gain, fp32 [H]
    // workspace for one chunk of up to kDecodeMaxRows rows
    h16_t *xa = nullptr;         // bf16: (x * g) as compact hi/lo operand
    float *ssq = nullptr;         // bf16: sums of squares per 16 columns
    float *x32 = nullptr, *n32 = nullptr;      // f32: x = a + b, normalised rows
    float *logits = nullptr;      // [rows][Vpad]
    float *scratch = nullptr;     // split partial sums of the batched projection
    size_t scratch_floats = 0;
};

namespace {
void free_head(hexgen_head *hd) {
    void *ptrs[] = {hd->w, hd->g, hd->xa, hd->ssq, hd->x32, hd->n32, hd->logits, hd->scratch};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
}
}  // namespace

hexgen_status_t hexgen_head_create(int hidden, int vocab, int tp_degree, int tp_rank, hexgen_dtype_t dtype, float rms_eps,
                                   hexgen_head_t **out) {
    if (!out) return HEXGEN_ERR_INVALID_ARG;
    *out = nullptr;
    if (hidden <= 0 || vocab <= 0 || tp_degree <= 0 || !(rms_eps >= 0.f)) return HEXGEN_ERR_INVALID_ARG;
    if (!known_dtype(dtype)) return HEXGEN_ERR_INVALID_ARG;
    if (tp_rank < 0 || tp_rank >= tp_degree || vocab % tp_degree) return HEXGEN_ERR_SHAPE;
    if (is_h16(dtype) && hidden % 128) return HEXGEN_ERR_SHAPE;
    if (dtype == HEXGEN_F32 && hidden % 4) return HEXGEN_ERR_SHAPE;
    hexgen_head *hd = new (std::nothrow) hexgen_head();
    if (!hd) return HEXGEN_ERR_OOM;
    hd->H = hidden; hd->V = vocab; hd->t = tp_degree; hd->r = tp_rank; hd->dtype = dtype; hd->eps = rms_eps;
    hd->Vl = vocab / tp_degree;
    hd->Vpad = round_up(hd->Vl, 16);
    const size_t rows = kDecodeMaxRows;
    hexgen_status_t rc = dmalloc(&hd->g, (size_t)hidden);
    if (rc == HEXGEN_OK) rc = dmalloc(&hd->logits, rows * hd->Vpad);
    if (rc == HEXGEN_OK && is_h16(dtype)) {
        rc = dmalloc(&hd->xa, 2 * rows * hidden);
        if (rc == HEXGEN_OK) rc = dmalloc(&hd->ssq, (size_t)(hidden / 16) * DEC_SSQ_STRIDE);
        hd->scratch_floats = rows * ((size_t)512 * 128 + 2 * (size_t)hd->Vpad);
        if (rc == HEXGEN_OK) rc = dmalloc(&hd->scratch, hd->scratch_floats);
    } else if (rc == HEXGEN_OK) {
        rc = dmalloc(&hd->x32, rows * hidden);
        if (rc == HEXGEN_OK) rc = dmalloc(&hd->n32, rows * hidden);
    }
    if (rc != HEXGEN_OK) { free_head(hd); delete hd; (void)hipGetLastError(); return rc == HEXGEN_ERR_DEVICE ? HEXGEN_ERR_OOM : rc; }
    *out = hd;
    return HEXGEN_OK;
}

void hexgen_head_destroy(hexgen_head_t *hd) {
    if (!hd) return;
    (void)hipDeviceSynchronize();
    free_head(hd);
    delete hd;
}

hexgen_status_t hexgen_head_load(hexgen_head_t *hd, const void *g_final, const void *w_lm) {
    if (!hd || !g_final || !w_lm) return HEXGEN_ERR_INVALID_ARG;
    HX_HIP(hipDeviceSynchronize());
    const int H = hd->H, c0 = hd->r * hd->Vl;
    const size_t es = esize(hd->dtype);
    if (hd->w) { (void)hipFree(hd->w); hd->w = nullptr; }
    hd->loaded = false;
    if (hd->dtype == HEXGEN_F32) {
        HX_HIP(hipMemcpy(hd->g, g_final, sizeof(float) * H, hipMemcpyDefault));
        HX_HIP(hipMalloc(&hd->w, (size_t)H * hd->Vl * es));
        HX_HIP(hipMemcpy2D(hd->w, (size_t)hd->Vl * es, static_cast<const char *>(w_lm) + (size_t)c0 * es, (size_t)hd->V * es,
                           (size_t)hd->Vl * es, H, hipMemcpyDefault));
    } else {
        // gain -> fp32; the rank's columns -> a dense zero-padded device matrix -> MFMA fragment tiles
        h16_t *tmp = nullptr;
        HX_TRY(dmalloc(&tmp, (size_t)H * hd->Vpad + H));
        hipError_t e = hipMemset(tmp, 0, ((size_t)H * hd->Vpad + H) * es);
        if (e == hipSuccess) e = hipMemcpy(tmp + (size_t)H * hd->Vpad, g_final, (size_t)H * es, hipMemcpyDefault);
        if (e == hipSuccess)
            e = hipMemcpy2D(tmp, (size_t)hd->Vpad * es, static_cast<const char *>(w_lm) + (size_t)c0 * es, (size_t)hd->V * es,
                            (size_t)hd->Vl * es, H, hipMemcpyDefault);
        if (e == hipSuccess) e = hipMalloc(&hd->w, (size_t)H * hd->Vpad * es);
        if (e == hipSuccess) {
            HX_K(hd->dtype, launch_cvt_h16_to_f32, tmp + (size_t)H * hd->Vpad, hd->g, H, nullptr);
            launch_pack_weight(tmp, hd->Vpad, 0, 0, H, hd->Vpad, static_cast<h16_t *>(hd->w), 0, 1, hd->Vpad / 16, 0, nullptr);
            e = hipDeviceSynchronize();
        }
        (void)hipFree(tmp);
        if (e != hipSuccess) { (void)hipGetLastError(); return HEXGEN_ERR_DEVICE; }
    }
    hd->loaded = true;
    return HEXGEN_OK;
}

hexgen_status_t hexgen_head_greedy(hexgen_head_t *hd, const void *hidden_a, const void *hidden_b, int n_rows,
                                   int32_t *token_out, float *logit_out, void *stream) {
    if (!hd || !hidden_a || !token_out || n_rows <= 0) return HEXGEN_ERR_INVALID_ARG;
    if (!hd->loaded) return HEXGEN_ERR_STATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t es = esize(hd->dtype);
    const int H = hd->H;
    for (int r0 = 0; r0 < n_rows; r0 += kDecodeMaxRows) {
        const int n = std::min(kDecodeMaxRows, n_rows - r0);
        const char *a = static_cast<const char *>(hidden_a) + (size_t)r0 * H * es;
        const char *b = hidden_b ? static_cast<const char *>(hidden_b) + (size_t)r0 * H * es : nullptr;
        int64_t ld = hd->Vpad;
        if (is_h16(hd->dtype)) {
            // same kernels as a decode projection: prologue (x = a + b, x * g as hi/lo operand, sums of squares),
            // weight-streaming projection with 1 / rms applied after the contraction, fp32 logits
            HX_K(hd->dtype, launch_decode_prologue, a, b, 1, nullptr, hd->g, hd->xa, hd->ssq, n, H, nullptr, nullptr, 0, s);
            DecodeEpi e;
            std::memset(&e, 0, sizeof(e));
            e.mode = DEC_RAW;
            e.ssq_in = hd->ssq;
            e.ssq_units = H / 16;
            e.norm_dim = H;
            e.eps = hd->eps;
            e.raw_out = hd->logits;
            HX_K(hd->dtype, launch_decode_proj, static_cast<const h16_t *>(hd->w), hd->xa, hd->Vpad, H, n, e, hd->scratch, hd->scratch_floats, s);
        } else {
            HX_HIP(hipMemcpyAsync(hd->x32, a, (size_t)n * H * es, hipMemcpyDeviceToDevice, s));
            if (b) launch_accumulate_f32(hd->x32, reinterpret_cast<const float *>(b), (int64_t)n * H, s);
            f32_launch_rmsnorm(hd->x32, hd->g, hd->n32, n, H, hd->eps, s);
            f32_launch_gemm(hd->n32, static_cast<const float *>(hd->w), hd->logits, n, H, hd->Vl, s);
            ld = hd->Vl;
        }
        launch_row_argmax(hd->logits, ld, hd->Vl, n, hd->r * hd->Vl, token_out + r0, logit_out ? logit_out + r0 : nullptr, s);
    }
    HX_HIP(hipGetLastError());
    return HEXGEN_OK;
}

hexgen_status_t hexgen_embed_rows(const void *table, hexgen_dtype_t dtype, int hidden, int vocab, const int32_t *tokens,
                                  int n, void *rows_out, void *stream) {
    if (!table || !tokens || !rows_out || hidden <= 0 || vocab <= 0 || n < 0) return HEXGEN_ERR_INVALID_ARG;
    if (!known_dtype(dtype)) return HEXGEN_ERR_INVALID_ARG;
    const int64_t row_bytes = (int64_t)hidden * (int64_t)esize(dtype);
    if (row_bytes % 4) return HEXGEN_ERR_SHAPE;
    launch_embed_rows(table, row_bytes, vocab, tokens, n, rows_out, static_cast<hipStream_t>(stream));
    HX_HIP(hipGetLastError());
    return HEXGEN_OK;
}

hexgen_status_t hexgen_set_attn_split(int nsplit) {
    if (nsplit < 0 || nsplit > kStaticAttnSplit) return HEXGEN_ERR_INVALID_ARG;
    g_attn_split_forced = nsplit;
    return HEXGEN_OK;
}

hexgen_status_t hexgen_set_gemm_tile(int code) {
    const bool a = bf16::set_gemm_tile(code), b = f16::set_gemm_tile(code);
    return a && b ? HEXGEN_OK : HEXGEN_ERR_INVALID_ARG;
}

hexgen_status_t hexgen_stage_set_tap(hexgen_stage_t *st, int layer, void *h_dump) {
    if (!st || layer < 0 || layer >= st->L) return HEXGEN_ERR_INVALID_ARG;
    st->taps[layer] = h_dump;
    return HEXGEN_OK;
}

}  // extern "C"
