// The verify engine behind the C ABI: argument validation, device memory plan, weight loading and the three
// orchestrations (verify prefill, prefill that returns states, token-by-token decode).  Host code only; all
// arithmetic of the method lives in the kernels this file launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "common.h"
#include "kernels.h"

using namespace vl;

namespace {

thread_local std::string g_create_error;

constexpr int64_t ALIGN = 256;
inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

std::string fmt(const char* f, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, f);
    vsnprintf(buf, sizeof(buf), f, ap);
    va_end(ap);
    return std::string(buf);
}

// ------------------------------------------------------------------------------------------------
// configuration checks and the memory plan (pure host arithmetic)
// ------------------------------------------------------------------------------------------------
bool check_cfg(const vl_model_cfg* c, std::string& why) {
    if (!c) { why = "cfg is NULL"; return false; }
    if (c->dtype != VL_F32 && c->dtype != VL_BF16) { why = "dtype must be VL_F32 or VL_BF16"; return false; }
    if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1 || c->d_ffn < 1 ||
        c->vocab < 1) { why = "model dimensions must be positive"; return false; }
    if (c->n_q_heads % c->n_kv_heads != 0) { why = "n_q_heads must be a multiple of n_kv_heads"; return false; }
    if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) { why = "rms_eps must be > 0 and rope_base > 1"; return false; }
    if (c->max_tokens < 1 || c->max_seqs < 1 || c->max_seq_len < 1) { why = "max_tokens/max_seqs/max_seq_len must be >= 1"; return false; }
    const int64_t qd = (int64_t)c->n_q_heads * c->head_dim;
    if (c->dtype == VL_BF16) {
        if (c->d_model % 64 || qd % 64 || c->d_ffn % 64) { why = "bf16 models need d_model, n_q_heads*head_dim, d_ffn multiples of 64"; return false; }
        if (c->head_dim != 128 && c->head_dim != 64) { why = "bf16 models need head_dim 64 or 128"; return false; }
        if (!attn_mfma_fits(c->n_q_heads, c->n_kv_heads, c->head_dim, c->max_seq_len)) {
            why = "max_seq_len too large: the q/k/v rows of one sequence must span less than 4 GB"; return false;
        }
    } else {
        if (c->d_model % 8 || c->d_ffn % 16 || c->head_dim % 4 || c->head_dim > 256) {
            why = "f32 models need d_model % 8 == 0, d_ffn % 16 == 0, head_dim % 4 == 0, head_dim <= 256"; return false;
        }
    }
    return true;
}

struct Plan {
    int64_t esz, d, qd, kvd, qkv_w, F, V, L, N, B, T, ib;
    int64_t layer_bytes, off_attn_norm, off_wqkv, off_wo, off_ffn_norm, off_wgu, off_wd;
    int64_t embed_bytes, lm_bytes, weights_total;
    int64_t vt_ld, max_tiles, stage_ints;
    int64_t workspace_total;
    // bf16 models keep every GEMM operand as a tiled image (see tiled_off): row counts padded to whole 256-row blocks
    int64_t Np, qkv_wp, dp, gup, Vp, wstage_bytes;
};

Plan make_plan(const vl_model_cfg& c) {
    Plan p{};
    p.esz = c.dtype == VL_BF16 ? 2 : 4;
    p.d = c.d_model; p.qd = (int64_t)c.n_q_heads * c.head_dim; p.kvd = (int64_t)c.n_kv_heads * c.head_dim;
    p.qkv_w = p.qd + 2 * p.kvd; p.F = c.d_ffn; p.V = c.vocab; p.L = c.n_layers;
    p.N = c.max_tokens; p.B = c.max_seqs; p.T = c.max_seq_len;
    p.ib = c.dtype == VL_BF16 ? 32 : 16;
    const bool tiled = c.dtype == VL_BF16;
    auto pr = [&](int64_t rows) { return tiled ? align_up(rows, TL_ROWS) : rows; };
    p.Np = pr(p.N); p.qkv_wp = pr(p.qkv_w); p.dp = pr(p.d); p.gup = pr(2 * p.F); p.Vp = pr(p.V);
    p.wstage_bytes = tiled ? (int64_t)64 << 20 : 0;
    int64_t o = 0;
    p.off_attn_norm = o; o = align_up(o + p.d * 4, ALIGN);
    p.off_wqkv = o; o = align_up(o + p.qkv_wp * p.d * p.esz, ALIGN);
    p.off_wo = o; o = align_up(o + p.dp * p.qd * p.esz, ALIGN);
    p.off_ffn_norm = o; o = align_up(o + p.d * 4, ALIGN);
    p.off_wgu = o; o = align_up(o + p.gup * p.d * p.esz, ALIGN);
    p.off_wd = o; o = align_up(o + p.dp * p.F * p.esz, ALIGN);
    p.layer_bytes = o;
    p.embed_bytes = align_up(p.V * p.d * p.esz, ALIGN);
    p.lm_bytes = align_up(p.Vp * p.d * p.esz, ALIGN);
    p.weights_total = p.layer_bytes * p.L + p.embed_bytes + p.lm_bytes + align_up(p.d * 4, ALIGN);
    // values transposed for the matrix-core attention: every sequence starts on a multiple of 8 columns, plus one
    // key tile of slack so that the last tile of the last sequence can be read whole
    p.vt_ld = align_up(p.N + 8 * p.B + 64, 64);
    p.max_tiles = p.N / 64 + p.B + 1;
    p.stage_ints = 12 * p.N + 6 * p.max_tiles + 8 * p.B + 64;
    int64_t w = 0;
    w += align_up(p.N * p.d * 4, ALIGN);                 // residual stream (fp32)
    w += align_up(p.Np * std::max(p.d, p.qd) * p.esz, ALIGN);  // normalised rows / attention output share nothing: two buffers
    w += align_up(p.Np * p.qd * p.esz, ALIGN);           // attention output
    w += align_up(p.N * p.qkv_w * p.esz, ALIGN);         // q | k | v
    w += align_up(p.Np * p.F * p.esz, ALIGN);            // silu(gate) * up
    w += align_up(p.wstage_bytes, ALIGN);                // staging for re-tiling weights as they are loaded
    w += align_up(p.N * p.V * 4, ALIGN);                 // logits (fp32)
    if (c.dtype == VL_BF16) w += align_up(p.kvd * p.vt_ld * 2, ALIGN);
    w += 2 * align_up(p.L * p.N * p.kvd * p.esz, ALIGN);   // KV cache of the decode path (packed like the tokens)
    w += align_up(p.T * (c.head_dim / 2) * 8, ALIGN);    // rotary cos/sin table
    w += align_up(p.stage_ints * 4, ALIGN);              // per-call index arrays
    w += align_up((int64_t)p.L * p.N * (int64_t)sizeof(vl_tok_stats), ALIGN);
    w += align_up((int64_t)p.L * p.N * (int64_t)sizeof(vl_bit_stats), ALIGN);
    w += align_up((int64_t)VL_MERKLE_MAX_OPENINGS * 2 * p.d * 32, ALIGN);
    w += 3 * align_up(p.N, ALIGN) + align_up(p.N * 4, ALIGN) * 2 + ALIGN;   // ok bytes, argmax, gap, summary
    p.workspace_total = w;
    return p;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// the context
// ------------------------------------------------------------------------------------------------
struct vl_ctx {
    vl_model_cfg cfg{};
    Plan plan{};
    int device = 0;
    hipStream_t stream = nullptr;
    bool capturing = false;             // a decode step is being recorded as a graph: no timing events
    bool own_stream = false;            // created here because the caller passed none (graphs cannot be captured on the NULL stream)
    std::string err;
    bool bf16 = false;

    std::vector<char*> layer_slab;      // one allocation per layer
    char* embed = nullptr;
    char* lm_head = nullptr;
    float* final_norm = nullptr;
    std::vector<uint8_t> loaded;        // [L][VL_T_COUNT] + globals at layer 0

    float* resid = nullptr;
    char* xn = nullptr;
    char* attn = nullptr;
    char* qkv = nullptr;
    char* act = nullptr;
    char* wstage = nullptr;             // bf16 models: row-major chunk of a weight tensor on its way to the tiled image
    float* logits = nullptr;
    char* vt = nullptr;
    char* kcache = nullptr;
    char* vcache = nullptr;
    float2* rope_cs = nullptr;
    int32_t* d_idx = nullptr;           // device copy of the per-call index arrays
    int32_t* h_idx = nullptr;           // pinned host staging for them
    vl_tok_stats* stats = nullptr;
    vl_bit_stats* bit_stats = nullptr;  // [L][N], written only while a bit rule is set
    uint32_t* merkle_scratch = nullptr; // VL_MERKLE_MAX_OPENINGS x 2 x d_model digests, for inclusion proofs
    bool has_rule = false;
    vl_bit_rule rule{};
    int last_bits_c = 0;                // committed layers of the most recent verify call that ran the rule
    uint8_t* hid_ok = nullptr;
    uint8_t* tok_ok = nullptr;
    uint8_t* scratch_ok = nullptr;
    int32_t* argmax = nullptr;
    float* gap = nullptr;
    DevSummary* d_summary = nullptr;
    DevSummary* h_summary = nullptr;    // pinned
    std::vector<void*> allocs;
    std::vector<hipEvent_t> events;

    int64_t last_n = 0;
    bool last_has_logits = false;
    int64_t logits_rows = 0;                                // rows of the most recent call whose logits are in `logits`

    // optional per-stage timing (vl_profile_enable): event pairs recorded around launches, read after the sync
    struct Span { int stage; hipEvent_t a, b; };
    int prof_mode = 0;
    std::vector<hipEvent_t> prof_pool;
    size_t prof_used = 0;
    std::vector<Span> prof_spans;
    double prof_ms[VL_STAGE_COUNT] = {};
    int64_t prof_launches[VL_STAGE_COUNT] = {};

    int fail(int code, const std::string& m) { err = m; return code; }
};

namespace {
// Records an event pair around the launches made while it is alive, if profiling covers `stage`.
struct StageSpan {
    vl_ctx* c; bool on = false; vl_ctx::Span sp{};
    StageSpan(vl_ctx* c_, int stage) : c(c_) {
        if (c->prof_mode == 0 || (c->prof_mode == 1 && stage != VL_STAGE_GATEUP_GEMM) || c->capturing) return;
        if (c->prof_used + 2 > c->prof_pool.size()) return;
        sp.stage = stage; sp.a = c->prof_pool[c->prof_used++]; sp.b = c->prof_pool[c->prof_used++];
        on = hipEventRecord(sp.a, c->stream) == hipSuccess;
    }
    ~StageSpan() {
        if (on && hipEventRecord(sp.b, c->stream) == hipSuccess) c->prof_spans.push_back(sp);
    }
};
void collect_profile(vl_ctx* c) {          // call after the stream has been synchronised
    for (auto& sp : c->prof_spans) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, sp.a, sp.b) == hipSuccess) { c->prof_ms[sp.stage] += t; c->prof_launches[sp.stage]++; }
    }
    c->prof_spans.clear();
    c->prof_used = 0;
}
}  // namespace

#define HIP_TRY(ctx, call)                                                                         \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return (ctx)->fail(e_ == hipErrorOutOfMemory ? VL_E_NOMEM : VL_E_HIP,                  \
                               fmt("%s failed: %s", #call, hipGetErrorString(e_)));                \
    } while (0)

namespace {

template <typename T>
int dev_alloc(vl_ctx* c, T** out, int64_t bytes, bool zero) {
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, (size_t)std::max<int64_t>(bytes, 16));
    if (e != hipSuccess) return c->fail(VL_E_NOMEM, fmt("hipMalloc(%lld bytes) failed: %s", (long long)bytes, hipGetErrorString(e)));
    c->allocs.push_back(p);
    if (zero) {
        e = hipMemset(p, 0, (size_t)std::max<int64_t>(bytes, 16));
        if (e != hipSuccess) return c->fail(VL_E_HIP, fmt("hipMemset failed: %s", hipGetErrorString(e)));
    }
    *out = (T*)p;
    return VL_OK;
}

bool all_loaded(const vl_ctx* c) {
    for (uint8_t v : c->loaded) if (!v) return false;
    return true;
}

// The tensors a pass over blocks lo+1 .. hi touches: those blocks, the embedding if it starts from tokens, the final
// norm and LM head if it ends with the token check.
bool range_loaded(const vl_ctx* c, int lo, int hi, bool embed, bool head) {
    for (int l = lo; l < hi; ++l)
        for (int k = 0; k < VL_T_COUNT; ++k)
            if (k != VL_T_EMBED && k != VL_T_FINAL_NORM && k != VL_T_LM_HEAD && !c->loaded[(size_t)l * VL_T_COUNT + k]) return false;
    if (embed && !c->loaded[VL_T_EMBED]) return false;
    if (head && (!c->loaded[VL_T_FINAL_NORM] || !c->loaded[VL_T_LM_HEAD])) return false;
    return true;
}

struct LayerW { float* attn_norm; char* wqkv; char* wo; float* ffn_norm; char* wgu; char* wd; };
LayerW layer_w(const vl_ctx* c, int l) {
    char* s = c->layer_slab[l];
    const Plan& p = c->plan;
    return {(float*)(s + p.off_attn_norm), s + p.off_wqkv, s + p.off_wo, (float*)(s + p.off_ffn_norm), s + p.off_wgu, s + p.off_wd};
}

// Index arrays of one packed batch, laid out back to back in the staging buffer.
struct BatchIdx {
    int64_t rows = 0;
    int32_t* pos = nullptr;         // position of the row in its sequence
    int32_t* seq_row0 = nullptr;    // first row (of this batch's qkv buffer) of the row's sequence
    int32_t* vt_col = nullptr;      // column of the row in the transposed-values buffer
    AttnTile* tiles = nullptr;
    int n_tiles = 0;
};

// Carves `count` ints out of the staging area; host and device views advance together.
struct Stage {
    int32_t* h; int32_t* d; int64_t used = 0, cap;
    Stage(int32_t* h_, int32_t* d_, int64_t cap_) : h(h_), d(d_), cap(cap_) {}
    bool take(int64_t count, int32_t** hp, int32_t** dp) {
        count = align_up(count, 4);
        if (used + count > cap) return false;
        *hp = h + used; *dp = d + used; used += count;
        return true;
    }
};

// Builds pos / seq_row0 / vt_col / tiles (one per q_span queries; none if q_span = 0) for sequences of the given
// lengths packed back to back.
bool build_batch_idx(Stage& st, const std::vector<int32_t>& lens, int q_span, BatchIdx* dev) {
    const bool want_tiles = q_span > 0;
    int64_t n = 0;
    for (int32_t t : lens) n += t;
    int32_t *hp, *hs, *hv;
    if (!st.take(n, &hp, &dev->pos) || !st.take(n, &hs, &dev->seq_row0) || !st.take(n, &hv, &dev->vt_col)) return false;
    std::vector<AttnTile> tiles;
    int64_t row = 0, col = 0;
    for (int32_t t : lens) {
        for (int32_t i = 0; i < t; ++i) {
            hp[row + i] = i;
            hs[row + i] = (int32_t)row;
            hv[row + i] = (int32_t)(col + i);
        }
        if (want_tiles)
            for (int32_t q0 = 0; q0 < t; q0 += q_span) {
                const int32_t qr = std::min(q_span, t - q0);
                tiles.push_back({(int32_t)(row + q0), qr, (int32_t)row, q0 + qr, (int32_t)col, q0});
            }
        row += t;
        col = align_up(col + t, 8);
    }
    dev->rows = n;
    dev->n_tiles = (int)tiles.size();
    if (want_tiles) {
        // longest first: the tiles with the most keys start first and the short ones fill the tail
        std::stable_sort(tiles.begin(), tiles.end(), [](const AttnTile& a, const AttnTile& b) { return a.kv_len > b.kv_len; });
        int32_t *ht, *dt;
        if (!st.take((int64_t)tiles.size() * 6, &ht, &dt)) return false;
        if (!tiles.empty()) memcpy(ht, tiles.data(), tiles.size() * sizeof(AttnTile));
        dev->tiles = (AttnTile*)dt;
    }
    return true;
}

// Queries per attention tile of this model's prefill (0: the fp32 path builds no tiles).
int attn_span(const vl_ctx* c) { return c->bf16 ? attn_mfma_q_span(c->cfg.n_q_heads, c->cfg.n_kv_heads) : 0; }

// bf16 models: every GEMM runs on the matrix cores; up to 64 rows (a decode step) take the weight-streaming kernel,
// more rows the 256 x 256 tile kernel.  fp32 models: vector-ALU GEMM.
void gemm(vl_ctx* c, const void* A, const void* W, int M, int N, int K, int epi, void* out) {
    // inside the engine every bf16 GEMM operand is a tiled image, and so is the SwiGLU output (the next GEMM's operand)
    const int layout = GL_A_TILED | GL_W_TILED | (epi == EPI_SWIGLU ? GL_OUT_TILED : 0);
    if (c->bf16 && M <= GEMM_SKINNY_MAX_M) launch_gemm_skinny(A, W, M, N, K, epi, out, c->stream, layout);
    else if (c->bf16) launch_gemm_mfma(A, W, M, N, K, epi, out, c->stream, layout);
    else launch_gemm_simple(A, W, c->cfg.dtype, M, N, K, epi, out, (int)c->plan.ib, c->stream);
}

// One decoder block over `rows` packed rows that form whole sequences (prefill form).
void block_prefill(vl_ctx* c, int l, const BatchIdx& bi, const int32_t* cache_row) {
    const vl_model_cfg& m = c->cfg;
    const Plan& p = c->plan;
    const LayerW w = layer_w(c, l);
    const int rows = (int)bi.rows;
    hipStream_t s = c->stream;
    { StageSpan sp(c, VL_STAGE_NORM); launch_rmsnorm(c->resid, w.attn_norm, c->xn, m.dtype, rows, m.d_model, m.rms_eps, s, c->bf16); }
    { StageSpan sp(c, VL_STAGE_QKV_GEMM); gemm(c, c->xn, w.wqkv, rows, (int)p.qkv_w, m.d_model, EPI_STORE, c->qkv); }
    {
        StageSpan sp(c, VL_STAGE_ROPE);
        const int64_t lo = (int64_t)l * p.N * p.kvd * p.esz;
        launch_rope(c->qkv, m.dtype, bi.pos, c->rope_cs, rows, m.n_q_heads, m.n_kv_heads, m.head_dim, s,
                    cache_row ? c->kcache + lo : nullptr, cache_row ? c->vcache + lo : nullptr, cache_row);
        if (c->bf16) launch_transpose_v(c->qkv, c->vt, bi.vt_col, rows, m.n_q_heads, m.n_kv_heads, m.head_dim, p.vt_ld, s);
    }
    {
        StageSpan sp(c, VL_STAGE_ATTENTION);
        if (c->bf16) {
            launch_attn_mfma(c->qkv, rows, c->vt, p.vt_ld, bi.tiles, bi.n_tiles, c->attn, m.n_q_heads, m.n_kv_heads, m.head_dim, s, true);
        } else {
            const char* q = c->qkv;
            launch_attn_rowwise(q, p.qkv_w, q + p.qd * p.esz, q + (p.qd + p.kvd) * p.esz, p.qkv_w, bi.seq_row0, bi.pos, c->attn,
                                m.dtype, rows, m.n_q_heads, m.n_kv_heads, m.head_dim, s);
        }
    }
    { StageSpan sp(c, VL_STAGE_O_GEMM); gemm(c, c->attn, w.wo, rows, m.d_model, (int)p.qd, EPI_ADD_RESID, c->resid); }
    { StageSpan sp(c, VL_STAGE_NORM); launch_rmsnorm(c->resid, w.ffn_norm, c->xn, m.dtype, rows, m.d_model, m.rms_eps, s, c->bf16); }
    { StageSpan sp(c, VL_STAGE_GATEUP_GEMM); gemm(c, c->xn, w.wgu, rows, 2 * m.d_ffn, m.d_model, EPI_SWIGLU, c->act); }
    { StageSpan sp(c, VL_STAGE_DOWN_GEMM); gemm(c, c->act, w.wd, rows, m.d_model, m.d_ffn, EPI_ADD_RESID, c->resid); }
}

// One decoder block over `rows` single positions, each attending to its sequence's KV cache (decode form).
void block_decode(vl_ctx* c, int l, int rows, const int32_t* pos, const int32_t* cache_row, const int32_t* cache_row0) {
    const vl_model_cfg& m = c->cfg;
    const Plan& p = c->plan;
    const LayerW w = layer_w(c, l);
    hipStream_t s = c->stream;
    const int64_t lo = (int64_t)l * p.N * p.kvd * p.esz;
    // few rows: the first RMSNorm runs inside the projection that consumes it
    const bool fuse_norm = c->bf16 && gemm_skinny_norm_supported(rows, m.d_model) && gemm_skinny_qkv_rope_supported(rows, m.head_dim);
    if (fuse_norm) {
        launch_gemm_skinny_qkv_rope(c->resid, w.wqkv, rows, m.d_model, c->qkv, pos, c->rope_cs, cache_row, c->kcache + lo, c->vcache + lo,
                                    m.n_q_heads, m.n_kv_heads, m.head_dim, s, GL_W_TILED, (const float*)w.attn_norm, m.rms_eps);
    } else {
        launch_rmsnorm(c->resid, w.attn_norm, c->xn, m.dtype, rows, m.d_model, m.rms_eps, s, c->bf16);
        if (c->bf16 && gemm_skinny_qkv_rope_supported(rows, m.head_dim)) {
            launch_gemm_skinny_qkv_rope(c->xn, w.wqkv, rows, m.d_model, c->qkv, pos, c->rope_cs, cache_row, c->kcache + lo,
                                        c->vcache + lo, m.n_q_heads, m.n_kv_heads, m.head_dim, s, GL_A_TILED | GL_W_TILED);
        } else {
            gemm(c, c->xn, w.wqkv, rows, (int)p.qkv_w, m.d_model, EPI_STORE, c->qkv);
            launch_rope(c->qkv, m.dtype, pos, c->rope_cs, rows, m.n_q_heads, m.n_kv_heads, m.head_dim, s, c->kcache + lo, c->vcache + lo,
                        cache_row);
        }
    }
    if (c->bf16 && attn_decode_supported(m.n_q_heads, m.n_kv_heads, m.head_dim))
        launch_attn_decode(c->qkv, p.qkv_w, c->kcache + lo, c->vcache + lo, p.kvd, cache_row0, pos, c->attn, rows, m.n_q_heads,
                           m.n_kv_heads, m.head_dim, s, true);
    else
        launch_attn_rowwise(c->qkv, p.qkv_w, c->kcache + lo, c->vcache + lo, p.kvd, cache_row0, pos, c->attn, m.dtype, rows,
                            m.n_q_heads, m.n_kv_heads, m.head_dim, s, c->bf16);
    gemm(c, c->attn, w.wo, rows, m.d_model, (int)p.qd, EPI_ADD_RESID, c->resid);
    launch_rmsnorm(c->resid, w.ffn_norm, c->xn, m.dtype, rows, m.d_model, m.rms_eps, s, c->bf16);
    gemm(c, c->xn, w.wgu, rows, 2 * m.d_ffn, m.d_model, EPI_SWIGLU, c->act);
    gemm(c, c->act, w.wd, rows, m.d_model, m.d_ffn, EPI_ADD_RESID, c->resid);
}

void lm_head_logits(vl_ctx* c, int rows) {
    const vl_model_cfg& m = c->cfg;
    { StageSpan sp(c, VL_STAGE_NORM); launch_rmsnorm(c->resid, c->final_norm, c->xn, m.dtype, rows, m.d_model, m.rms_eps, c->stream, c->bf16); }
    { StageSpan sp(c, VL_STAGE_LM_GEMM); gemm(c, c->xn, c->lm_head, rows, m.vocab, m.d_model, EPI_STORE_F32, c->logits); }
    c->logits_rows = rows;
}

// Final norm, LM head, argmax and token check of `rows` rows.  With more rows than the weight-streaming GEMM takes, the
// argmax is the epilogue of the LM-head GEMM and the logits are never written (their buffer holds the per-part maxima;
// vl_get_logits recomputes them on demand from the normalised rows, which stay in xn).
// ea / eb (optional) are recorded around the argmax part.
int lm_head_argmax(vl_ctx* c, int rows, const int32_t* committed, float margin, float* gap, uint8_t* tok_ok, hipEvent_t ea = nullptr,
                   hipEvent_t eb = nullptr) {
    const vl_model_cfg& m = c->cfg;
    hipStream_t s = c->stream;
    const int64_t ld = rows, parts = argmax_parts(m.vocab);
    const bool fused = c->bf16 && rows > GEMM_SKINNY_MAX_M && (parts * ld * 8 + ld * 4) <= c->plan.N * c->plan.V * 4;
    if (!fused) {
        lm_head_logits(c, rows);
        if (ea) HIP_TRY(c, hipEventRecord(ea, s));
        {
            StageSpan sp(c, VL_STAGE_ARGMAX);
            launch_argmax(c->logits, rows, m.vocab, committed, margin, c->argmax, gap, tok_ok, s);
        }
        if (eb) HIP_TRY(c, hipEventRecord(eb, s));
        return VL_OK;
    }
    { StageSpan sp(c, VL_STAGE_NORM); launch_rmsnorm(c->resid, c->final_norm, c->xn, m.dtype, rows, m.d_model, m.rms_eps, s, c->bf16); }
    ArgmaxParts ap{c->logits, (int32_t*)c->logits + parts * ld, committed, c->logits + 2 * parts * ld, ld};
    {
        StageSpan sp(c, VL_STAGE_LM_GEMM);
        launch_gemm_mfma_argmax(c->xn, c->lm_head, rows, m.vocab, m.d_model, ap, s, GL_A_TILED | GL_W_TILED);
    }
    if (ea) HIP_TRY(c, hipEventRecord(ea, s));
    {
        StageSpan sp(c, VL_STAGE_ARGMAX);
        launch_argmax_reduce(ap, rows, m.vocab, committed, margin, c->argmax, gap, tok_ok, s);
    }
    if (eb) HIP_TRY(c, hipEventRecord(eb, s));
    c->logits_rows = 0;
    return VL_OK;
}

int check_batch(vl_ctx* c, const int32_t* tokens, const int32_t* lengths, int32_t B, const int32_t* commit_layers, int32_t C,
                int32_t hidden_dtype, int64_t* n_out, bool whole_model = true) {
    if (!c) return VL_E_ARG;
    if (B < 0 || (B > 0 && !lengths)) return c->fail(VL_E_ARG, "lengths is NULL or B < 0");
    if (C < 0 || (C > 0 && !commit_layers)) return c->fail(VL_E_ARG, "commit_layers is NULL or C < 0");
    if (hidden_dtype != VL_F32 && hidden_dtype != VL_BF16) return c->fail(VL_E_ARG, "hidden_dtype must be VL_F32 or VL_BF16");
    if (B > c->cfg.max_seqs) return c->fail(VL_E_CAPACITY, fmt("B = %d exceeds max_seqs = %d", B, c->cfg.max_seqs));
    int64_t n = 0;
    for (int b = 0; b < B; ++b) {
        if (lengths[b] < 0) return c->fail(VL_E_ARG, fmt("lengths[%d] is negative", b));
        if (lengths[b] > c->cfg.max_seq_len)      // positions index the rotary table
            return c->fail(VL_E_CAPACITY, fmt("lengths[%d] = %d exceeds max_seq_len = %d", b, lengths[b], c->cfg.max_seq_len));
        n += lengths[b];
    }
    if (n > c->cfg.max_tokens) return c->fail(VL_E_CAPACITY, fmt("N = %lld exceeds max_tokens = %d", (long long)n, c->cfg.max_tokens));
    for (int i = 0; i < C; ++i) {
        if (commit_layers[i] < 1 || commit_layers[i] > c->cfg.n_layers) return c->fail(VL_E_ARG, fmt("commit_layers[%d] = %d outside [1, %d]", i, commit_layers[i], c->cfg.n_layers));
        if (i > 0 && commit_layers[i] <= commit_layers[i - 1]) return c->fail(VL_E_ARG, "commit_layers must be strictly ascending");
    }
    if (whole_model) {
        if (n > 0 && !tokens) return c->fail(VL_E_ARG, "tokens is NULL");
        if (!all_loaded(c)) return c->fail(VL_E_WEIGHTS, "not every weight tensor has been loaded");
    }
    *n_out = n;
    return VL_OK;
}

int upload_stage(vl_ctx* c, const Stage& st) {
    if (st.used > 0) HIP_TRY(c, hipMemcpyAsync(c->d_idx, c->h_idx, (size_t)st.used * 4, hipMemcpyHostToDevice, c->stream));
    return VL_OK;
}

// A pass that covers only blocks start_layer+1 .. end_layer and, for start_layer > 0, begins from recorded states.
struct Segment { int start_layer, end_layer; const void* upstream_hidden; int upstream_dtype; };

// The shared prefill driver: compare against commitments (verify) or write the states out (commit).
int run_prefill(vl_ctx* c, const int32_t* tokens, const int32_t* lengths, int32_t B, const int32_t* commit_layers, int32_t C,
                const void* committed_hidden, void* out_hidden, int32_t hidden_dtype, const int32_t* committed_argmax,
                int32_t* out_argmax, bool run_head, const vl_tol* tol, uint8_t* flags, vl_tok_stats* stats_out,
                vl_summary* summary, bool verify, const Segment* seg = nullptr) {
    int64_t n = 0;
    int rc = check_batch(c, tokens, lengths, B, commit_layers, C, hidden_dtype, &n, seg == nullptr);
    if (rc) return rc;
    const int layer_lo = seg ? seg->start_layer : 0, layer_hi = seg ? seg->end_layer : c->cfg.n_layers;
    const bool from_tokens = !seg || seg->start_layer == 0;
    if (seg) {
        if (layer_lo < 0 || layer_hi > c->cfg.n_layers || layer_lo >= layer_hi)
            return c->fail(VL_E_ARG, fmt("segment (%d, %d] is not a non-empty layer range inside [0, %d]", layer_lo, layer_hi, c->cfg.n_layers));
        for (int i = 0; i < C; ++i)
            if (commit_layers[i] <= layer_lo || commit_layers[i] > layer_hi)
                return c->fail(VL_E_ARG, fmt("commit_layers[%d] = %d outside the segment (%d, %d]", i, commit_layers[i], layer_lo, layer_hi));
        if (run_head && layer_hi != c->cfg.n_layers) return c->fail(VL_E_ARG, "the token check needs a segment that ends at the last layer");
        if (seg->upstream_dtype != VL_F32 && seg->upstream_dtype != VL_BF16) return c->fail(VL_E_ARG, "upstream_dtype must be VL_F32 or VL_BF16");
        if (n > 0 && from_tokens && !tokens) return c->fail(VL_E_ARG, "tokens is NULL for a segment that starts at the embedding");
        if (n > 0 && !from_tokens && !seg->upstream_hidden) return c->fail(VL_E_ARG, "upstream_hidden is NULL");
        if (!range_loaded(c, layer_lo, layer_hi, from_tokens, run_head))
            return c->fail(VL_E_WEIGHTS, "a weight tensor this segment needs has not been loaded");
    }
    HIP_TRY(c, hipSetDevice(c->device));
    c->last_n = 0;
    c->last_has_logits = false;
    c->last_bits_c = 0;
    if (summary) memset(summary, 0, sizeof(*summary));
    if (n == 0) return VL_OK;
    if (verify && C > 0 && !committed_hidden) return c->fail(VL_E_ARG, "committed_hidden is NULL");
    if (verify && !flags) return c->fail(VL_E_ARG, "flags is NULL");
    const vl_model_cfg& m = c->cfg;
    const int rows = (int)n;
    hipStream_t s = c->stream;
    // the previous call synchronised before returning, so the staging buffer is free
    Stage st(c->h_idx, c->d_idx, c->plan.stage_ints);
    BatchIdx bi;
    std::vector<int32_t> lens(lengths, lengths + B);
    if (!build_batch_idx(st, lens, attn_span(c), &bi)) return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    rc = upload_stage(c, st);
    if (rc) return rc;

    size_t ev = 0;
    float ms_compare = 0.f;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> cmp_spans;
    hipEvent_t e_start = c->events[ev++], e_stop = c->events[ev++];
    HIP_TRY(c, hipEventRecord(e_start, s));
    if (verify) {
        launch_fill_u8(c->hid_ok, 1, n, s);
        launch_fill_u8(c->tok_ok, 1, n, s);
    }
    {
        StageSpan sp(c, VL_STAGE_EMBED);
        if (from_tokens) launch_embed(c->embed, m.dtype, tokens, nullptr, c->resid, verify ? c->hid_ok : nullptr, nullptr, n, m.d_model, m.vocab, s);
        else launch_load_hidden(seg->upstream_hidden, seg->upstream_dtype, c->resid, n, m.d_model, s);
    }
    int ci = 0;
    for (int l = layer_lo; l < layer_hi; ++l) {
        block_prefill(c, l, bi, nullptr);
        if (ci < C && commit_layers[ci] == l + 1) {
            const int64_t off = (int64_t)ci * n * m.d_model * (hidden_dtype == VL_BF16 ? 2 : 4);
            if (verify) {
                hipEvent_t a = c->events[ev++], b = c->events[ev++];
                HIP_TRY(c, hipEventRecord(a, s));
                {
                    StageSpan sp(c, VL_STAGE_COMPARE);
                    launch_compare(c->resid, (const char*)committed_hidden + off, hidden_dtype, n, m.d_model, tol->rel_l2, tol->max_abs,
                                   c->stats + (int64_t)ci * n, c->hid_ok, nullptr, s, c->has_rule ? &c->rule : nullptr,
                                   c->bit_stats + (int64_t)ci * n);
                }
                HIP_TRY(c, hipEventRecord(b, s));
                cmp_spans.push_back({a, b});
            } else if (out_hidden) {
                launch_store_hidden(c->resid, (char*)out_hidden + off, hidden_dtype, nullptr, n, m.d_model, s);
            }
            ++ci;
        }
    }
    if (run_head) {
        hipEvent_t a = c->events[ev++], b = c->events[ev++];
        const int hrc = lm_head_argmax(c, rows, verify ? committed_argmax : nullptr, verify ? tol->logit_margin : 0.f, c->gap,
                                       verify ? c->tok_ok : nullptr, a, b);
        if (hrc) return hrc;
        cmp_spans.push_back({a, b});
        if (!verify && out_argmax) HIP_TRY(c, hipMemcpyAsync(out_argmax, c->argmax, (size_t)n * 4, hipMemcpyDeviceToDevice, s));
    }
    if (verify) {
        hipEvent_t a = c->events[ev++], b = c->events[ev++];
        HIP_TRY(c, hipEventRecord(a, s));
        { StageSpan sp(c, VL_STAGE_FINALIZE); launch_finalize(c->hid_ok, c->tok_ok, c->stats, C, n, flags, c->d_summary, s); }
        HIP_TRY(c, hipEventRecord(b, s));
        cmp_spans.push_back({a, b});
        if (stats_out && C > 0)
            HIP_TRY(c, hipMemcpyAsync(stats_out, c->stats, (size_t)C * n * sizeof(vl_tok_stats), hipMemcpyDeviceToDevice, s));
        HIP_TRY(c, hipMemcpyAsync(c->h_summary, c->d_summary, sizeof(DevSummary), hipMemcpyDeviceToHost, s));
    }
    HIP_TRY(c, hipEventRecord(e_stop, s));
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(s));
    collect_profile(c);
    c->last_n = n;
    c->last_has_logits = run_head;
    c->last_bits_c = (verify && c->has_rule) ? C : 0;
    if (summary) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, e_start, e_stop));
        for (auto& sp : cmp_spans) {
            float t = 0.f;
            HIP_TRY(c, hipEventElapsedTime(&t, sp.first, sp.second));
            ms_compare += t;
        }
        summary->n_tokens = n;
        summary->ms_forward = ms;
        summary->ms_compare = ms_compare;
        if (verify) {
            summary->n_rejected = (int64_t)c->h_summary->n_rejected;
            summary->n_hidden_reject = (int64_t)c->h_summary->n_hidden_reject;
            summary->n_token_reject = (int64_t)c->h_summary->n_token_reject;
            summary->max_rel_l2 = c->h_summary->max_rel;
            summary->max_abs = c->h_summary->max_abs;
            summary->mean_mae = c->h_summary->mean_mae;
        }
    }
    return VL_OK;
}

}  // namespace

// ================================================================================================
// C ABI
// ================================================================================================
extern "C" {

int vl_plan_memory(const vl_model_cfg* cfg, uint64_t* weight_bytes, uint64_t* workspace_bytes) {
    std::string why;
    if (!check_cfg(cfg, why)) { g_create_error = why; return VL_E_ARG; }
    const Plan p = make_plan(*cfg);
    if (weight_bytes) *weight_bytes = (uint64_t)p.weights_total;
    if (workspace_bytes) *workspace_bytes = (uint64_t)p.workspace_total;
    return VL_OK;
}

const char* vl_last_error(const vl_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

void vl_destroy(vl_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)(ctx->stream ? hipStreamSynchronize(ctx->stream) : hipDeviceSynchronize());
    for (void* p : ctx->allocs) (void)hipFree(p);
    for (hipEvent_t e : ctx->events) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->prof_pool) (void)hipEventDestroy(e);
    if (ctx->h_idx) (void)hipHostFree(ctx->h_idx);
    if (ctx->h_summary) (void)hipHostFree(ctx->h_summary);
    if (ctx->own_stream) (void)hipStreamDestroy(ctx->stream);
    delete ctx;
}

int vl_create(const vl_model_cfg* cfg, int device, void* hip_stream, vl_ctx** out) {
    if (out) *out = nullptr;
    std::string why;
    if (!out) { g_create_error = "out is NULL"; return VL_E_ARG; }
    if (!check_cfg(cfg, why)) { g_create_error = why; return VL_E_ARG; }
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev < 1) { g_create_error = fmt("no HIP device available (%s)", hipGetErrorString(e)); return VL_E_HIP; }
    if (device < 0 || device >= ndev) { g_create_error = fmt("device %d out of range [0, %d)", device, ndev); return VL_E_ARG; }
    e = hipSetDevice(device);
    if (e != hipSuccess) { g_create_error = fmt("hipSetDevice failed: %s", hipGetErrorString(e)); return VL_E_HIP; }

    vl_ctx* c = new (std::nothrow) vl_ctx();
    if (!c) { g_create_error = "out of host memory"; return VL_E_NOMEM; }
    c->cfg = *cfg;
    c->plan = make_plan(*cfg);
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    if (!c->stream) {
        // default flags and default priority: the stream still orders itself against the NULL stream, like the NULL
        // stream itself would, so callers that produce inputs there need no extra synchronisation
        e = hipStreamCreate(&c->stream);
        if (e != hipSuccess) { g_create_error = fmt("hipStreamCreate failed: %s", hipGetErrorString(e)); delete c; return VL_E_HIP; }
        c->own_stream = true;
    }
    c->bf16 = cfg->dtype == VL_BF16;
    const Plan& p = c->plan;
    int rc = VL_OK;
    auto bail = [&](int code) { g_create_error = c->err; vl_destroy(c); return code; };

    c->layer_slab.resize(p.L, nullptr);
    for (int64_t l = 0; l < p.L; ++l)
        if ((rc = dev_alloc(c, &c->layer_slab[l], p.layer_bytes, c->bf16))) return bail(rc);   // padding rows of tiled images = 0
    if ((rc = dev_alloc(c, &c->embed, p.embed_bytes, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->lm_head, p.lm_bytes, c->bf16))) return bail(rc);
    if ((rc = dev_alloc(c, &c->final_norm, p.d * 4, false))) return bail(rc);
    c->loaded.assign((size_t)p.L * VL_T_COUNT, 0);
    for (int64_t l = 1; l < p.L; ++l)      // the three global tensors are tracked at layer 0 only
        c->loaded[l * VL_T_COUNT + VL_T_EMBED] = c->loaded[l * VL_T_COUNT + VL_T_FINAL_NORM] = c->loaded[l * VL_T_COUNT + VL_T_LM_HEAD] = 1;

    if ((rc = dev_alloc(c, &c->resid, p.N * p.d * 4, false))) return bail(rc);
    // zeroed: rows past the batch (up to the next multiple of 256) are read by the GEMM tiles and must stay finite
    if ((rc = dev_alloc(c, &c->xn, p.Np * std::max(p.d, p.qd) * p.esz, true))) return bail(rc);
    if ((rc = dev_alloc(c, &c->attn, p.Np * p.qd * p.esz, true))) return bail(rc);
    if (p.wstage_bytes && (rc = dev_alloc(c, &c->wstage, p.wstage_bytes, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->qkv, p.N * p.qkv_w * p.esz, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->act, p.Np * p.F * p.esz, true))) return bail(rc);
    if ((rc = dev_alloc(c, &c->logits, p.N * p.V * 4, false))) return bail(rc);
    if (c->bf16 && (rc = dev_alloc(c, &c->vt, p.kvd * p.vt_ld * 2, true))) return bail(rc);   // zeroed: padding columns are read
    if ((rc = dev_alloc(c, &c->kcache, p.L * p.N * p.kvd * p.esz, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->vcache, p.L * p.N * p.kvd * p.esz, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->rope_cs, p.T * (cfg->head_dim / 2) * 8, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->d_idx, p.stage_ints * 4, true))) return bail(rc);
    if ((rc = dev_alloc(c, &c->stats, p.L * p.N * (int64_t)sizeof(vl_tok_stats), false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->bit_stats, p.L * p.N * (int64_t)sizeof(vl_bit_stats), false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->merkle_scratch, (int64_t)VL_MERKLE_MAX_OPENINGS * 2 * p.d * 32, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->hid_ok, p.N, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->tok_ok, p.N, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->scratch_ok, p.N, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->argmax, p.N * 4, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->gap, p.N * 4, false))) return bail(rc);
    if ((rc = dev_alloc(c, &c->d_summary, sizeof(DevSummary), true))) return bail(rc);
    if (hipHostMalloc((void**)&c->h_idx, (size_t)p.stage_ints * 4, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc((void**)&c->h_summary, sizeof(DevSummary), hipHostMallocDefault) != hipSuccess) {
        c->err = "hipHostMalloc failed";
        return bail(VL_E_NOMEM);
    }
    c->events.resize(2 * (size_t)p.L + 8);
    for (auto& ev : c->events)
        if (hipEventCreate(&ev) != hipSuccess) { c->err = "hipEventCreate failed"; ev = nullptr; return bail(VL_E_HIP); }

    // rotary table: angle = pos * base^(-2i/head_dim) evaluated in double, cos/sin rounded once to float
    {
        const int half = cfg->head_dim / 2;
        std::vector<float2> tab((size_t)p.T * half);
        for (int64_t t = 0; t < p.T; ++t)
            for (int i = 0; i < half; ++i) {
                const double ang = (double)t * std::pow((double)cfg->rope_base, -2.0 * i / (double)cfg->head_dim);
                tab[(size_t)t * half + i] = make_float2((float)std::cos(ang), (float)std::sin(ang));
            }
        if (hipMemcpy(c->rope_cs, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice) != hipSuccess) {
            c->err = "upload of the rotary table failed";
            return bail(VL_E_HIP);
        }
    }
    *out = c;
    return VL_OK;
}

int vl_load_weights(vl_ctx* c, int kind, int layer, const void* src, size_t nbytes) {
    if (!c) return VL_E_ARG;
    if (!src) return c->fail(VL_E_ARG, "src is NULL");
    if (kind < 0 || kind >= VL_T_COUNT) return c->fail(VL_E_ARG, fmt("tensor_kind %d out of range", kind));
    const bool global = kind == VL_T_EMBED || kind == VL_T_FINAL_NORM || kind == VL_T_LM_HEAD;
    if (global) layer = 0;
    if (layer < 0 || layer >= c->cfg.n_layers) return c->fail(VL_E_ARG, fmt("layer %d out of range [0, %d)", layer, c->cfg.n_layers));
    const Plan& p = c->plan;
    int64_t want = 0;
    switch (kind) {
        case VL_T_EMBED: case VL_T_LM_HEAD: want = p.V * p.d * p.esz; break;
        case VL_T_ATTN_NORM: case VL_T_FFN_NORM: case VL_T_FINAL_NORM: want = p.d * 4; break;
        case VL_T_WQ: want = p.qd * p.d * p.esz; break;
        case VL_T_WK: case VL_T_WV: want = p.kvd * p.d * p.esz; break;
        case VL_T_WO: want = p.d * p.qd * p.esz; break;
        case VL_T_W_GATE: case VL_T_W_UP: case VL_T_W_DOWN: want = p.F * p.d * p.esz; break;
    }
    if ((int64_t)nbytes != want) return c->fail(VL_E_ARG, fmt("tensor kind %d needs %lld bytes, got %zu", kind, (long long)want, nbytes));
    HIP_TRY(c, hipSetDevice(c->device));
    hipStream_t s = c->stream;
    const LayerW w = layer_w(c, layer);
    char* dst = nullptr;
    switch (kind) {
        case VL_T_EMBED: dst = c->embed; break;
        case VL_T_LM_HEAD: dst = c->lm_head; break;
        case VL_T_FINAL_NORM: dst = (char*)c->final_norm; break;
        case VL_T_ATTN_NORM: dst = (char*)w.attn_norm; break;
        case VL_T_FFN_NORM: dst = (char*)w.ffn_norm; break;
        case VL_T_WQ: dst = w.wqkv; break;                                       // fused [q | k | v] rows
        case VL_T_WK: dst = w.wqkv + p.qd * p.d * p.esz; break;
        case VL_T_WV: dst = w.wqkv + (p.qd + p.kvd) * p.d * p.esz; break;
        case VL_T_WO: dst = w.wo; break;
        case VL_T_W_DOWN: dst = w.wd; break;
        default: break;
    }
    const bool matrix = kind != VL_T_EMBED && kind != VL_T_ATTN_NORM && kind != VL_T_FFN_NORM && kind != VL_T_FINAL_NORM;
    if (c->bf16 && matrix) {
        // GEMM operands of a bf16 model are stored as tiled images (see tiled_off): the tensor passes through a
        // row-major staging buffer in chunks of whole 32-row blocks and a kernel scatters each chunk into place
        int64_t rows = 0, K = 0, row0 = 0;
        char* image = nullptr;
        int interleave = 0;
        switch (kind) {
            case VL_T_WQ: image = w.wqkv; rows = p.qd; K = p.d; break;                  // fused [q | k | v] rows
            case VL_T_WK: image = w.wqkv; rows = p.kvd; K = p.d; row0 = p.qd; break;
            case VL_T_WV: image = w.wqkv; rows = p.kvd; K = p.d; row0 = p.qd + p.kvd; break;
            case VL_T_WO: image = w.wo; rows = p.d; K = p.qd; break;
            case VL_T_W_DOWN: image = w.wd; rows = p.d; K = p.F; break;
            case VL_T_LM_HEAD: image = c->lm_head; rows = p.V; K = p.d; break;
            // rows interleaved in blocks of 32: [gate 0..32) | up 0..32) | gate 32..64) | ...] so that a GEMM tile holds
            // gate and up of the same channels and can apply SwiGLU in its epilogue
            case VL_T_W_GATE: image = w.wgu; rows = p.F; K = p.d; interleave = 1; break;
            default: image = w.wgu; rows = p.F; K = p.d; interleave = 2; break;
        }
        const int64_t row_bytes = K * 2;
        const int64_t chunk = std::max<int64_t>(32, (p.wstage_bytes / row_bytes) / 32 * 32);
        if (chunk * row_bytes > p.wstage_bytes) return c->fail(VL_E_CAPACITY, "a 32-row block of this tensor exceeds the staging buffer");
        for (int64_t r = 0; r < rows; r += chunk) {
            const int64_t nr = std::min(chunk, rows - r);
            HIP_TRY(c, hipMemcpyAsync(c->wstage, (const char*)src + r * row_bytes, (size_t)(nr * row_bytes), hipMemcpyDefault, s));
            // chunks start on multiples of 32 rows, so the interleaving of a chunk is that of its first row plus an offset
            launch_retile(c->wstage, image, nr, (int)K, interleave ? row0 + 2 * r : row0 + r, interleave, s);
            HIP_TRY(c, hipGetLastError());
            HIP_TRY(c, hipStreamSynchronize(s));                // the staging buffer is reused by the next chunk
        }
    } else if (kind == VL_T_W_GATE || kind == VL_T_W_UP) {
        // rows interleaved in blocks of ib: [gate 0..ib) | up 0..ib) | gate ib..2ib) | ...] so that a GEMM tile
        // holds gate and up of the same channels and can apply SwiGLU in its epilogue
        const size_t blk = (size_t)(p.ib * p.d * p.esz);
        char* base = w.wgu + (kind == VL_T_W_UP ? blk : 0);
        HIP_TRY(c, hipMemcpy2DAsync(base, 2 * blk, src, blk, blk, (size_t)(p.F / p.ib), hipMemcpyDefault, s));
    } else {
        HIP_TRY(c, hipMemcpyAsync(dst, src, nbytes, hipMemcpyDefault, s));
    }
    HIP_TRY(c, hipStreamSynchronize(s));
    c->loaded[(size_t)layer * VL_T_COUNT + kind] = 1;
    return VL_OK;
}

int vl_verify_prefill(vl_ctx* c, const int32_t* tokens, const int32_t* lengths, int32_t B, const int32_t* commit_layers,
                      int32_t C, const void* committed_hidden, int32_t hidden_dtype, const int32_t* committed_argmax,
                      const vl_tol* tol, uint8_t* flags, vl_tok_stats* stats, vl_summary* summary) {
    if (!c) return VL_E_ARG;
    if (!tol) return c->fail(VL_E_ARG, "tol is NULL");
    return run_prefill(c, tokens, lengths, B, commit_layers, C, committed_hidden, nullptr, hidden_dtype, committed_argmax, nullptr,
                       committed_argmax != nullptr, tol, flags, stats, summary, true);
}

int vl_verify_segment(vl_ctx* c, int32_t start_layer, int32_t end_layer, const void* upstream_hidden, int32_t upstream_dtype,
                      const int32_t* tokens, const int32_t* lengths, int32_t B, const int32_t* commit_layers, int32_t C,
                      const void* committed_hidden, int32_t hidden_dtype, const int32_t* committed_argmax, const vl_tol* tol,
                      uint8_t* flags, vl_tok_stats* stats, vl_summary* summary) {
    if (!c) return VL_E_ARG;
    if (!tol) return c->fail(VL_E_ARG, "tol is NULL");
    const Segment seg{start_layer, end_layer, upstream_hidden, upstream_dtype};
    return run_prefill(c, tokens, lengths, B, commit_layers, C, committed_hidden, nullptr, hidden_dtype, committed_argmax, nullptr,
                       committed_argmax != nullptr, tol, flags, stats, summary, true, &seg);
}

namespace {
bool rule_valid(const vl_bit_rule* r) {
    const float f[] = {r->e_w, r->q_small, r->tau_large, r->pe_max, r->pm_min, r->pw_min, r->eps_max, r->q_small_min, r->z_large_max};
    for (float v : f) if (v != v) return false;
    return r->e_m >= 0 && r->step_log2 >= 0 && r->step_log2 <= 23;
}
}  // namespace

int vl_set_bit_rule(vl_ctx* c, const vl_bit_rule* rule) {
    if (!c) return VL_E_ARG;
    if (rule && !rule_valid(rule)) return c->fail(VL_E_ARG, "bit rule: e_m must be >= 0, step_log2 within [0, 23], no field NaN");
    c->has_rule = rule != nullptr;
    if (rule) c->rule = *rule;
    return VL_OK;
}

int vl_get_bit_stats(vl_ctx* c, int32_t ci, int64_t tok_begin, int64_t tok_end, vl_bit_stats* out) {
    if (!c) return VL_E_ARG;
    if (c->last_bits_c == 0) return c->fail(VL_E_ARG, "the most recent call ran no bit-aware rule");
    if (ci < 0 || ci >= c->last_bits_c || tok_begin < 0 || tok_end < tok_begin || tok_end > c->last_n)
        return c->fail(VL_E_ARG, "commit-layer index or token range outside the most recent verify call");
    if (tok_end == tok_begin) return VL_OK;
    if (!out) return c->fail(VL_E_ARG, "out is NULL");
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, hipMemcpyAsync(out, c->bit_stats + (int64_t)ci * c->last_n + tok_begin, (size_t)(tok_end - tok_begin) * sizeof(vl_bit_stats),
                              hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_prefill_commit(vl_ctx* c, const int32_t* tokens, const int32_t* lengths, int32_t B, const int32_t* commit_layers, int32_t C,
                      void* out_hidden, int32_t hidden_dtype, int32_t* out_argmax) {
    if (!c) return VL_E_ARG;
    return run_prefill(c, tokens, lengths, B, commit_layers, C, nullptr, out_hidden, hidden_dtype, nullptr, out_argmax,
                       out_argmax != nullptr, nullptr, nullptr, nullptr, nullptr, false);
}

int vl_decode_commit(vl_ctx* c, const int32_t* tokens, const int32_t* lengths, const int32_t* prompt_lens, int32_t B,
                     const int32_t* commit_layers, int32_t C, void* out_hidden, int32_t hidden_dtype, int32_t* out_argmax) {
    int64_t n = 0;
    int rc = check_batch(c, tokens, lengths, B, commit_layers, C, hidden_dtype, &n);
    if (rc) return rc;
    const vl_model_cfg& m = c->cfg;
    const Plan& p = c->plan;
    std::vector<int32_t> plen(B, 0);
    int32_t max_len = 0;
    for (int b = 0; b < B; ++b) {
        if (prompt_lens) plen[b] = prompt_lens[b];
        if (plen[b] < 0 || plen[b] > lengths[b]) return c->fail(VL_E_ARG, fmt("prompt_lens[%d] outside [0, lengths]", b));
        max_len = std::max(max_len, lengths[b]);
    }
    HIP_TRY(c, hipSetDevice(c->device));
    c->last_n = 0;
    c->last_has_logits = false;
    if (n == 0) return VL_OK;
    hipStream_t s = c->stream;
    const int64_t hsz = hidden_dtype == VL_BF16 ? 2 : 4;
    std::vector<int64_t> cu(B + 1, 0);
    for (int b = 0; b < B; ++b) cu[b + 1] = cu[b] + lengths[b];

    Stage st(c->h_idx, c->d_idx, p.stage_ints);
    // ---- prompt part: one prefill over the packed prompts, filling the KV cache
    BatchIdx bi;
    if (!build_batch_idx(st, plen, attn_span(c), &bi)) return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    const int64_t np = bi.rows;
    int32_t *h_src, *d_src, *h_crow, *d_crow;
    if (!st.take(np, &h_src, &d_src) || !st.take(np, &h_crow, &d_crow)) return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    {
        int64_t r = 0;
        for (int b = 0; b < B; ++b)
            for (int32_t t = 0; t < plen[b]; ++t, ++r) {
                h_src[r] = (int32_t)(cu[b] + t);                 // row in the caller's packed layout
                h_crow[r] = (int32_t)(cu[b] + t);                // row in the KV cache (packed like the tokens)
            }
    }
    // ---- decode part: step t handles every sequence with prompt_len <= t < length
    const int64_t nd = n - np;
    int32_t *h_dsrc, *d_dsrc, *h_dpos, *d_dpos, *h_dcrow, *d_dcrow, *h_dcrow0, *d_dcrow0;
    if (!st.take(nd, &h_dsrc, &d_dsrc) || !st.take(nd, &h_dpos, &d_dpos) || !st.take(nd, &h_dcrow, &d_dcrow) ||
        !st.take(nd, &h_dcrow0, &d_dcrow0))
        return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    int32_t *h_cur, *d_cur, *h_off, *d_off;             // per-step copies of the four index slices; running offset
    if (!st.take(4 * p.B, &h_cur, &d_cur) || !st.take(1, &h_off, &d_off)) return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    h_off[0] = 0;
    std::vector<std::pair<int64_t, int>> steps;        // (offset into the arrays, rows) per step
    {
        int64_t r = 0;
        for (int32_t t = 0; t < max_len; ++t) {
            const int64_t r0 = r;
            for (int b = 0; b < B; ++b)
                if (plen[b] <= t && t < lengths[b]) {
                    h_dsrc[r] = (int32_t)(cu[b] + t);
                    h_dpos[r] = t;
                    h_dcrow[r] = (int32_t)(cu[b] + t);
                    h_dcrow0[r] = (int32_t)cu[b];
                    ++r;
                }
            if (r > r0) steps.push_back({r0, (int)(r - r0)});
        }
    }
    rc = upload_stage(c, st);
    if (rc) return rc;

    auto emit = [&](int l, int rows, const int32_t* dst) {
        for (int ci = 0; ci < C; ++ci)
            if (commit_layers[ci] == l + 1 && out_hidden)
                launch_store_hidden(c->resid, (char*)out_hidden + (int64_t)ci * n * m.d_model * hsz, hidden_dtype, dst, rows, m.d_model, s);
    };
    if (np > 0) {
        launch_embed(c->embed, m.dtype, tokens, d_src, c->resid, nullptr, nullptr, np, m.d_model, m.vocab, s);
        for (int l = 0; l < m.n_layers; ++l) {
            block_prefill(c, l, bi, d_crow);
            emit(l, (int)np, d_src);
        }
        if (out_argmax) {
            lm_head_argmax(c, (int)np, nullptr, 0.f, nullptr, nullptr);
            launch_scatter_i32(c->argmax, out_argmax, d_src, np, s);
        }
    }
    // ---- decode steps.  Every step first copies its slice of the index arrays into fixed per-step buffers (and
    // advances a device-side offset), so all its launches have the same arguments as those of any other step with
    // the same number of live sequences: such a step is captured once as a graph and replayed, which removes the
    // ~260 host launches per step that otherwise bound the loop.
    auto run_step = [&](int rows) {
        launch_step_prologue(d_dsrc, d_dpos, d_dcrow, d_dcrow0, d_cur, d_off, rows, (int)p.B, s);
        const int32_t *cur_src = d_cur, *cur_pos = d_cur + p.B, *cur_crow = d_cur + 2 * p.B, *cur_crow0 = d_cur + 3 * p.B;
        launch_embed(c->embed, m.dtype, tokens, cur_src, c->resid, nullptr, nullptr, rows, m.d_model, m.vocab, s);
        for (int l = 0; l < m.n_layers; ++l) {
            block_decode(c, l, rows, cur_pos, cur_crow, cur_crow0);
            emit(l, rows, cur_src);
        }
        if (out_argmax) {
            lm_head_argmax(c, rows, nullptr, 0.f, nullptr, nullptr);
            launch_scatter_i32(c->argmax, out_argmax, cur_src, rows, s);
        }
    };
    std::vector<int> steps_with(p.B + 1, 0);
    for (auto& stp : steps) ++steps_with[stp.second];
    std::vector<hipGraphExec_t> execs(p.B + 1, nullptr);
    std::vector<hipGraph_t> graphs(p.B + 1, nullptr);
    auto drop_graphs = [&]() {
        for (auto& e : execs) if (e) { (void)hipGraphExecDestroy(e); e = nullptr; }
        for (auto& g : graphs) if (g) { (void)hipGraphDestroy(g); g = nullptr; }
    };
    constexpr int GRAPH_MIN_STEPS = 4;                          // below this an instantiation costs more than it saves
    for (auto& stp : steps) {
        const int rows = stp.second;
        if (steps_with[rows] < GRAPH_MIN_STEPS) { run_step(rows); continue; }
        if (!execs[rows]) {
            hipError_t e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
            if (e == hipSuccess) {
                c->capturing = true;
                run_step(rows);
                c->capturing = false;
                e = hipStreamEndCapture(s, &graphs[rows]);
            }
            if (e == hipSuccess) e = hipGraphInstantiate(&execs[rows], graphs[rows], nullptr, nullptr, 0);
            if (e != hipSuccess) {
                drop_graphs();
                return c->fail(VL_E_HIP, fmt("capturing a decode step as a graph failed: %s", hipGetErrorString(e)));
            }
        }
        const hipError_t e = hipGraphLaunch(execs[rows], s);
        if (e != hipSuccess) {
            drop_graphs();
            return c->fail(VL_E_HIP, fmt("hipGraphLaunch failed: %s", hipGetErrorString(e)));
        }
    }
    {
        const hipError_t e1 = hipGetLastError(), e2 = hipStreamSynchronize(s);
        drop_graphs();
        if (e1 != hipSuccess || e2 != hipSuccess)
            return c->fail(VL_E_HIP, fmt("decode steps failed: %s", hipGetErrorString(e1 != hipSuccess ? e1 : e2)));
    }
    return VL_OK;
}

int vl_get_logits(vl_ctx* c, int64_t tok_begin, int64_t tok_end, float* out) {
    if (!c) return VL_E_ARG;
    if (!c->last_has_logits) return c->fail(VL_E_ARG, "the most recent call ran no LM head");
    if (tok_begin < 0 || tok_end < tok_begin || tok_end > c->last_n) return c->fail(VL_E_ARG, "token range outside the most recent call");
    if (tok_end == tok_begin) return VL_OK;
    if (!out) return c->fail(VL_E_ARG, "out is NULL");
    HIP_TRY(c, hipSetDevice(c->device));
    const int64_t v = c->cfg.vocab;
    if (c->logits_rows < c->last_n) {                          // the call fused the argmax into the LM head: materialise them now
        gemm(c, c->xn, c->lm_head, (int)c->last_n, c->cfg.vocab, c->cfg.d_model, EPI_STORE_F32, c->logits);
        HIP_TRY(c, hipGetLastError());
        c->logits_rows = c->last_n;
    }
    HIP_TRY(c, hipMemcpyAsync(out, c->logits + tok_begin * v, (size_t)((tok_end - tok_begin) * v * 4), hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_get_argmax(vl_ctx* c, int64_t tok_begin, int64_t tok_end, int32_t* out_argmax, float* out_gap) {
    if (!c) return VL_E_ARG;
    if (!c->last_has_logits) return c->fail(VL_E_ARG, "the most recent call ran no LM head");
    if (tok_begin < 0 || tok_end < tok_begin || tok_end > c->last_n) return c->fail(VL_E_ARG, "token range outside the most recent call");
    if (tok_end == tok_begin) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t cnt = (size_t)(tok_end - tok_begin);
    if (out_argmax) HIP_TRY(c, hipMemcpyAsync(out_argmax, c->argmax + tok_begin, cnt * 4, hipMemcpyDeviceToDevice, c->stream));
    if (out_gap) HIP_TRY(c, hipMemcpyAsync(out_gap, c->gap + tok_begin, cnt * 4, hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_profile_enable(vl_ctx* c, int mode) {
    if (!c) return VL_E_ARG;
    if (mode < 0 || mode > 2) return c->fail(VL_E_ARG, "mode must be 0, 1 or 2");
    HIP_TRY(c, hipSetDevice(c->device));
    const size_t want = mode == 0 ? 0 : 2 * (size_t)(10 * c->cfg.n_layers + 16);
    while (c->prof_pool.size() < want) {
        hipEvent_t e;
        HIP_TRY(c, hipEventCreate(&e));
        c->prof_pool.push_back(e);
    }
    c->prof_mode = mode;
    return VL_OK;
}

int vl_profile_read(vl_ctx* c, double* ms, int64_t* launches) {
    if (!c) return VL_E_ARG;
    for (int i = 0; i < VL_STAGE_COUNT; ++i) {
        if (ms) ms[i] = c->prof_ms[i];
        if (launches) launches[i] = c->prof_launches[i];
        c->prof_ms[i] = 0.0;
        c->prof_launches[i] = 0;
    }
    return VL_OK;
}

int vl_op_gemm_bf16(vl_ctx* c, const void* A, const void* W, void* out, int32_t out_dtype, int32_t M, int32_t N, int32_t K) {
    if (!c) return VL_E_ARG;
    if (!A || !W || !out) return c->fail(VL_E_ARG, "A, W or out is NULL");
    if (M < 1 || N < 1 || K < 64 || K % 64) return c->fail(VL_E_ARG, "need M, N >= 1 and K a positive multiple of 64");
    if (out_dtype != VL_F32 && out_dtype != VL_BF16) return c->fail(VL_E_ARG, "out_dtype must be VL_F32 or VL_BF16");
    HIP_TRY(c, hipSetDevice(c->device));
    if (M <= GEMM_SKINNY_MAX_M) launch_gemm_skinny(A, W, M, N, K, out_dtype == VL_BF16 ? EPI_STORE : EPI_STORE_F32, out, c->stream);
    else launch_gemm_mfma(A, W, M, N, K, out_dtype == VL_BF16 ? EPI_STORE : EPI_STORE_F32, out, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_op_attention_bf16(vl_ctx* c, const void* qkv, const int32_t* lengths, int32_t B, void* out) {
    if (!c) return VL_E_ARG;
    if (!c->bf16) return c->fail(VL_E_ARG, "the context is not a bf16 model");
    if (!qkv || !out || !lengths || B < 0) return c->fail(VL_E_ARG, "qkv, out or lengths is NULL, or B < 0");
    if (B > c->cfg.max_seqs) return c->fail(VL_E_CAPACITY, "B exceeds max_seqs");
    int64_t n = 0;
    for (int b = 0; b < B; ++b) {
        if (lengths[b] < 0) return c->fail(VL_E_ARG, "negative length");
        n += lengths[b];
    }
    // (no positions are looked up here: rotary embedding is already applied by the caller)
    if (n > c->cfg.max_tokens) return c->fail(VL_E_CAPACITY, "N exceeds max_tokens");
    if (n == 0) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    const vl_model_cfg& m = c->cfg;
    Stage st(c->h_idx, c->d_idx, c->plan.stage_ints);
    BatchIdx bi;
    std::vector<int32_t> lens(lengths, lengths + B);
    if (!build_batch_idx(st, lens, attn_mfma_q_span(c->cfg.n_q_heads, c->cfg.n_kv_heads), &bi)) return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    int rc = upload_stage(c, st);
    if (rc) return rc;
    launch_transpose_v(qkv, c->vt, bi.vt_col, n, m.n_q_heads, m.n_kv_heads, m.head_dim, c->plan.vt_ld, c->stream);
    launch_attn_mfma(qkv, n, c->vt, c->plan.vt_ld, bi.tiles, bi.n_tiles, out, m.n_q_heads, m.n_kv_heads, m.head_dim, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_op_attention_decode_bf16(vl_ctx* c, const void* q, const void* k_cache, const void* v_cache, int64_t cache_rows,
                                const int32_t* first_row, const int32_t* n_keys, int32_t rows, void* out) {
    if (!c) return VL_E_ARG;
    if (!c->bf16) return c->fail(VL_E_ARG, "the context is not a bf16 model");
    const vl_model_cfg& m = c->cfg;
    if (!attn_decode_supported(m.n_q_heads, m.n_kv_heads, m.head_dim))
        return c->fail(VL_E_ARG, "needs head_dim 64 or 128 and n_q_heads / n_kv_heads in {1, 2, 4, 8}");
    if (rows < 0 || (rows > 0 && (!q || !k_cache || !v_cache || !first_row || !n_keys || !out)))
        return c->fail(VL_E_ARG, "NULL argument or rows < 0");
    for (int r = 0; r < rows; ++r)
        if (n_keys[r] < 1 || first_row[r] < 0 || (int64_t)first_row[r] + n_keys[r] > cache_rows)
            return c->fail(VL_E_ARG, fmt("row %d: keys [%d, %d + %d) outside the cache of %lld rows", r, first_row[r], first_row[r],
                                         n_keys[r], (long long)cache_rows));
    if (rows == 0) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    Stage st(c->h_idx, c->d_idx, c->plan.stage_ints);
    int32_t *h0, *d0, *hp, *dp;
    if (!st.take(rows, &h0, &d0) || !st.take(rows, &hp, &dp)) return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    for (int r = 0; r < rows; ++r) {
        h0[r] = first_row[r];
        hp[r] = n_keys[r] - 1;                                  // position of the query = index of its last key
    }
    int rc = upload_stage(c, st);
    if (rc) return rc;
    const int64_t kvd = (int64_t)m.n_kv_heads * m.head_dim;
    launch_attn_decode(q, (int64_t)m.n_q_heads * m.head_dim, k_cache, v_cache, kvd, d0, dp, out, rows, m.n_q_heads, m.n_kv_heads,
                       m.head_dim, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_op_compare(vl_ctx* c, const float* h_hat, const void* committed, int32_t hidden_dtype, int64_t N, const vl_tol* tol,
                  vl_tok_stats* stats, uint8_t* ok) {
    if (!c) return VL_E_ARG;
    if (N < 0 || (N > 0 && (!h_hat || !committed)) || !tol) return c->fail(VL_E_ARG, "bad pointer or N < 0");
    if (hidden_dtype != VL_F32 && hidden_dtype != VL_BF16) return c->fail(VL_E_ARG, "hidden_dtype must be VL_F32 or VL_BF16");
    if (N == 0) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    launch_compare(h_hat, committed, hidden_dtype, N, c->cfg.d_model, tol->rel_l2, tol->max_abs, stats, nullptr, ok, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_op_compare_bits(vl_ctx* c, const float* h_hat, const void* committed, int32_t hidden_dtype, int64_t N, const vl_tol* tol,
                       const vl_bit_rule* rule, vl_tok_stats* stats, vl_bit_stats* bits, uint8_t* ok) {
    if (!c) return VL_E_ARG;
    if (N < 0 || (N > 0 && (!h_hat || !committed)) || !tol || !rule) return c->fail(VL_E_ARG, "bad pointer or N < 0");
    if (hidden_dtype != VL_F32 && hidden_dtype != VL_BF16) return c->fail(VL_E_ARG, "hidden_dtype must be VL_F32 or VL_BF16");
    if (!rule_valid(rule)) return c->fail(VL_E_ARG, "bit rule: e_m must be >= 0, step_log2 within [0, 23], no field NaN");
    if (N == 0) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    launch_compare(h_hat, committed, hidden_dtype, N, c->cfg.d_model, tol->rel_l2, tol->max_abs, stats, nullptr, ok, c->stream, rule, bits);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_op_merkle_roots(vl_ctx* c, const void* states, int32_t dtype, int64_t rows, uint8_t* roots) {
    if (!c) return VL_E_ARG;
    if (rows < 0 || (rows > 0 && (!states || !roots))) return c->fail(VL_E_ARG, "bad pointer or rows < 0");
    if (dtype != VL_F32 && dtype != VL_BF16) return c->fail(VL_E_ARG, "dtype must be VL_F32 or VL_BF16");
    if (c->cfg.d_model > 16384) return c->fail(VL_E_CAPACITY, "Merkle trees are built for d_model <= 16384");
    if (rows > 0x7fffffff) return c->fail(VL_E_CAPACITY, "more than 2^31 - 1 rows in one call");
    if (rows == 0) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    launch_merkle_roots(states, dtype, rows, c->cfg.d_model, roots, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_op_merkle_open(vl_ctx* c, const void* states, int32_t dtype, int64_t rows, const int64_t* sel_row, const int32_t* sel_index,
                      int32_t K, float* values, uint8_t* paths, int32_t* path_len) {
    if (!c) return VL_E_ARG;
    if (K < 0 || (K > 0 && (!states || !sel_row || !sel_index || !paths))) return c->fail(VL_E_ARG, "bad pointer or K < 0");
    if (dtype != VL_F32 && dtype != VL_BF16) return c->fail(VL_E_ARG, "dtype must be VL_F32 or VL_BF16");
    if (K > VL_MERKLE_MAX_OPENINGS) return c->fail(VL_E_CAPACITY, fmt("K = %d exceeds VL_MERKLE_MAX_OPENINGS = %d", K, VL_MERKLE_MAX_OPENINGS));
    const int d = c->cfg.d_model;
    if (d > 16384) return c->fail(VL_E_CAPACITY, "Merkle trees are built for d_model <= 16384");
    for (int q = 0; q < K; ++q)
        if (sel_row[q] < 0 || sel_row[q] >= rows || sel_row[q] > 0x7fffffff || sel_index[q] < 0 || sel_index[q] >= d)
            return c->fail(VL_E_ARG, fmt("opening %d: row %lld / element %d outside [0, %lld) x [0, %d)", q, (long long)sel_row[q],
                                         sel_index[q], (long long)rows, d));
    if (K == 0) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    Stage st(c->h_idx, c->d_idx, c->plan.stage_ints);
    int32_t *hr, *dr, *hi, *di;
    if (!st.take(K, &hr, &dr) || !st.take(K, &hi, &di)) return c->fail(VL_E_CAPACITY, "index staging buffer too small");
    for (int q = 0; q < K; ++q) {
        hr[q] = (int32_t)sel_row[q];
        hi[q] = sel_index[q];
        if (path_len) {                                         // a level adds a digest iff the node has a sibling there
            int n = d, idx = sel_index[q], len = 0;
            while (n > 1) {
                if ((idx ^ 1) < n) ++len;
                idx >>= 1;
                n = (n + 1) >> 1;
            }
            path_len[q] = len;
        }
    }
    int rc = upload_stage(c, st);
    if (rc) return rc;
    launch_merkle_open(states, dtype, d, dr, di, K, c->merkle_scratch, paths, values, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

int vl_op_argmax(vl_ctx* c, const float* logits, int64_t N, const int32_t* committed_argmax, float margin, int32_t* out_argmax,
                 float* out_gap, uint8_t* out_ok) {
    if (!c) return VL_E_ARG;
    if (N < 0 || (N > 0 && !logits)) return c->fail(VL_E_ARG, "bad pointer or N < 0");
    if (N == 0) return VL_OK;
    HIP_TRY(c, hipSetDevice(c->device));
    launch_argmax(logits, N, c->cfg.vocab, committed_argmax, margin, out_argmax, out_gap, out_ok, c->stream);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return VL_OK;
}

}  // extern "C"
