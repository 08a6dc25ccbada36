// Host side of the C ABI declared in include/ssd.h: argument checks, the decoding state
// machine, the workspace carve-up and the per-layer launch sequences.  All arithmetic of the
// hot path lives in the kernels (ssd_kernels.hip); this file only orders them.
#include "../../include/ssd.h"
#include "ssd_kernels.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

using namespace ssdk;

namespace {

enum State { ST_CREATED = 0, ST_READY = 1, ST_IDLE = 2, ST_DRAFTED = 3, ST_VERIFIED = 4 };

constexpr size_t ALIGN = 256;
size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Layout {
    size_t rope, kv, x, h, qkv, att, act, part, logits, taps, tapn, hi, lo, ssq, small, vtok, ring, ring_conf, total;
    int rows;       // activation rows: max(max_k + 1, prompt rows per pass)
    int prefill_rows;  // prompt rows per pass: SSD_PREFILL_ROWS where the shape fits the 128 x 128 tiling, 64 where only the
                       // 64-row one, else 16
    int tap_rows;   // rows of the tap buffer: a verify block, or the 16 rows of a short prompt (a longer prompt keeps
                    // the taps of its last row only)
    int conf_rows;  // rows of one confidence pass: 2 * L
    int logit_rows;
    size_t kv_layer_elems;  // elements of K (or V) of one layer
    size_t part_floats;     // floats in the attention scratch (also the K-split scratch of the 64-row projections)
};

bool valid_cfg(const ssd_config* c)
{
    if (!c) return false;
    if (c->n_layers < 1 || c->n_layers > SSD_MAX_LAYERS || c->d_model < 16 || c->n_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 16 ||
        c->vocab < 16 || c->max_seq < 2)
        return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->n_heads % c->n_kv_heads) return false;
    long dq = (long)c->n_heads * c->head_dim, dkv = (long)c->n_kv_heads * c->head_dim;
    if (c->d_model % 16 || c->d_ffn % 16 || dq % 16 || dkv % 16 || c->vocab % 16) return false;
    if (c->weight_dtype < 0 || c->weight_dtype > 2) return false;
    if (c->kv_dtype < 0 || c->kv_dtype > 2) return false;
    if (c->conf_taps != 1 && c->conf_taps != 2) return false;
    if (c->max_k < 1 || c->max_k > SSD_MAX_K) return false;
    if (c->conf_window < 0 || c->conf_window > SSD_MAX_WINDOW) return false;
    if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f) || !(c->conf_clamp > 0.f) || !(c->conf_eps >= 0.f)) return false;
    return true;
}

Dims make_dims(const ssd_config& c)
{
    Dims D;
    D.L = c.n_layers; D.d = c.d_model; D.H = c.n_heads; D.Hkv = c.n_kv_heads; D.hd = c.head_dim;
    D.dq = c.n_heads * c.head_dim; D.dkv = c.n_kv_heads * c.head_dim; D.f = c.d_ffn; D.V = c.vocab;
    D.max_seq = c.max_seq; D.eps = c.rms_eps; D.wt = c.weight_dtype; D.kt = c.kv_dtype;
    return D;
}

Layout make_layout(const ssd_config& c)
{
    Dims D = make_dims(c);
    Layout l;
    size_t esz = c.kv_dtype == 0 ? 4 : 2;
    l.prefill_rows = rows_big_supported(D) ? SSD_PREFILL_ROWS : rows_wide_supported(D) ? 64 : 16;
    {   // no more rows per pass than a prompt can have (rounded up to whole 64-row groups)
        const int cap = (c.max_seq + 63) / 64 * 64;
        if (l.prefill_rows > 64 && l.prefill_rows > cap) l.prefill_rows = cap;
    }
    l.rows = c.max_k + 1 > l.prefill_rows ? c.max_k + 1 : l.prefill_rows;
    l.tap_rows = c.max_k + 1 > 16 ? c.max_k + 1 : 16;
    l.conf_rows = 2 * c.n_layers;
    l.logit_rows = l.rows > l.conf_rows ? l.rows : l.conf_rows;
    l.kv_layer_elems = (size_t)D.Hkv * D.max_seq * D.hd;
    size_t kmax = (size_t)(D.d > D.dq ? D.d : D.dq);
    size_t o = 0;
    l.rope = o;   o += align_up((size_t)D.max_seq * (D.hd / 2) * 2 * sizeof(float));
    l.kv = o;     o += align_up((size_t)D.L * 2 * l.kv_layer_elems * esz);
    l.x = o;      o += align_up((size_t)l.rows * D.d * sizeof(float));
    l.h = o;      o += align_up((size_t)l.rows * kmax * sizeof(float));
    l.qkv = o;    o += align_up((size_t)l.rows * (D.dq + 2 * D.dkv) * sizeof(float));
    l.att = o;    o += align_up((size_t)l.rows * D.dq * sizeof(float));
    l.act = o;    o += align_up((size_t)l.rows * D.f * sizeof(float));
    l.part_floats = attention_scratch_floats(D, l.rows);
    l.part = o;   o += align_up(l.part_floats * sizeof(float));
    l.logits = o; o += align_up((size_t)l.logit_rows * D.V * sizeof(float));
    l.taps = o;   o += align_up((size_t)l.tap_rows * D.L * 2 * D.d * sizeof(float));
    l.tapn = o;   o += align_up((size_t)l.conf_rows * D.d * sizeof(float));
    {   // bf16 hi/lo staging of activation rows for the MFMA path: rows x max(d, dq, f), or the confidence rows x d
        size_t kbig = (size_t)(D.f > (int)kmax ? D.f : (int)kmax);
        size_t a = (size_t)l.rows * kbig, b = (size_t)l.conf_rows * D.d;
        size_t n = a > b ? a : b;
        l.hi = o; o += align_up(n * 2);
        l.lo = o; o += align_up(n * 2);
    }
    l.ssq = o;    o += align_up((size_t)l.rows * (D.d / 16 + 1) * sizeof(float));  // per-tile sums of squares of the residual rows
    l.small = o;  o += align_up(4096);
    l.vtok = o;   o += align_up((size_t)l.rows * sizeof(int32_t));   // token ids of a prompt block
    // context window of the confidence extraction: hidden-state taps [window][2L][d] of the last `window` processed
    // positions, and one confidence value per tap row of the window
    l.ring = o;       o += align_up((size_t)c.conf_window * 2 * D.L * D.d * sizeof(float));
    l.ring_conf = o;  o += align_up(((size_t)c.conf_window * 2 * D.L + 2 * D.L) * sizeof(float));
    l.total = o;
    return l;
}

// offsets (in 4-byte words) inside the "small" region
enum { SM_POS = 0, SM_TOK = 8 /* 17 ints: pending + drafts */, SM_RES = 56 /* 2 */, SM_MAXPROB = 64 /* 16 floats */,
       SM_SINK = 96, SM_CONF = 128 /* conf_rows floats x3 follow (at most 3 x 2 x SSD_MAX_LAYERS, checked where used) */,
       SM_VTOK = 896 /* 64: tokens of a row block */, SM_TARGET = 960 /* 64: greedy token after each row of a block */ };

}  // namespace

struct ssd_ctx {
    ssd_config cfg;
    Dims D;
    LaunchOpts opts;   // D.opt points here
    Layout lay;
    hipStream_t stream;
    State state;
    std::string err;
    char* ws;
    size_t ws_bytes;
    bool have_w;
    ssd_weights w;
    std::vector<const float*> attn_norm, mlp_norm;
    std::vector<const void*> wq, wk, wv, wo, wg, wu, wd;
    int n;             // committed tokens
    int k_pending;     // k of the draft awaiting verification / acceptance
    int tap_rows;      // rows with valid taps (0 = none)
    long ring_count;   // positions pushed into the context-window ring since the last prefill
    int tap_row0;      // index of the first valid tap row inside the tap buffer
    int logit_rows;    // rows with valid logits
    int32_t* pinned;   // host-pinned readback buffer
    int device;        // device that was current when the workspace was set
    void* static_scratch;  // this device's copy of the library's static scratch array (resolved at set_workspace)
    ssd_stats st;
    bool use_graphs;   // replay captured launch sequences instead of launching kernel by kernel
    std::map<std::string, hipGraphExec_t> graphs;  // nullptr = sequence seen once, not captured yet
    int prof_kid;      // kernel id being timed, -1 = off
    size_t prof_used;  // event pairs in use
    std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_ev;

    float* f(size_t off) const { return reinterpret_cast<float*>(ws + off); }
    uint16_t* h16(size_t off) const { return reinterpret_cast<uint16_t*>(ws + off); }
    int32_t* small_i() const { return reinterpret_cast<int32_t*>(ws + lay.small); }
    float* small_f() const { return reinterpret_cast<float*>(ws + lay.small); }
    int* pos_dev() const { return small_i() + SM_POS; }
    void* kcache(int l) const
    {
        size_t esz = cfg.kv_dtype == 0 ? 4 : 2;
        return ws + lay.kv + ((size_t)l * 2 + 0) * lay.kv_layer_elems * esz;
    }
    void* vcache(int l) const
    {
        size_t esz = cfg.kv_dtype == 0 ? 4 : 2;
        return ws + lay.kv + ((size_t)l * 2 + 1) * lay.kv_layer_elems * esz;
    }
};

namespace {

int fail(ssd_ctx* c, int code, const char* msg)
{
    if (c) c->err = msg;
    return code;
}

int hip_fail(ssd_ctx* c, hipError_t e, const char* where)
{
    if (c) c->err = std::string(where) + ": " + hipGetErrorString(e);
    return SSD_EHIP;
}

#define HIPCHK(call, where)                                  \
    do {                                                     \
        hipError_t e__ = (call);                             \
        if (e__ != hipSuccess) return hip_fail(c, e__, where); \
    } while (0)

// the single-launch GEMV kernels can time themselves (events bound to the kernel's own timestamps)
static inline bool is_gemv_kid(int kid)
{
    return kid == SSD_K_GEMV_QKV || kid == SSD_K_GEMV_GATEUP || kid == SSD_K_GEMV_DOWN || kid == SSD_K_GEMV_LMHEAD;
}

// Launch `call`; when kernel `kid` is selected for timing, bracket it with a pair of events.
#define TIMED(kid, call, where)                                                            \
    do {                                                                                   \
        if (c->prof_kid == (kid)) {                                                        \
            if (c->prof_used == c->prof_ev.size()) {                                       \
                hipEvent_t a__, b__;                                                       \
                HIPCHK(hipEventCreate(&a__), "event create");                              \
                HIPCHK(hipEventCreate(&b__), "event create");                              \
                c->prof_ev.emplace_back(a__, b__);                                         \
            }                                                                              \
            if (is_gemv_kid(kid)) {                                                        \
                c->opts.time_start = c->prof_ev[c->prof_used].first;                       \
                c->opts.time_stop = c->prof_ev[c->prof_used].second;                       \
                HIPCHK(call, where);                                                       \
            } else {                                                                       \
                HIPCHK(hipEventRecord(c->prof_ev[c->prof_used].first, c->stream), "event"); \
                HIPCHK(call, where);                                                       \
                HIPCHK(hipEventRecord(c->prof_ev[c->prof_used].second, c->stream), "event"); \
            }                                                                              \
            c->prof_used++;                                                                \
        } else {                                                                           \
            HIPCHK(call, where);                                                           \
        }                                                                                  \
    } while (0)

// One decoder layer for a single row (draft / vanilla decode path); either sub-block may be left out.
int layer_single(ssd_ctx* c, int l, int pos_off, bool do_attn, bool do_mlp)
{
    const Dims& D = c->D;
    float* x = c->f(c->lay.x);
    if (do_attn) {
    TIMED(SSD_K_GEMV_QKV, gemv_qkv(D, c->wq[l], c->wk[l], c->wv[l], c->attn_norm[l], x, c->f(c->lay.rope), c->pos_dev(),
                                   pos_off, c->f(c->lay.qkv), c->kcache(l), c->vcache(l), c->stream), "gemv_qkv");
    int fold = 0;  // > 0: attention left that many partials per head for the output projection to fold
    TIMED(SSD_K_ATTENTION, attention(D, c->f(c->lay.qkv), D.dq, c->kcache(l), c->vcache(l), c->pos_dev(), pos_off,
                                     c->n - 1, 1, c->f(c->lay.part), c->f(c->lay.att), nullptr, nullptr, c->stream, &fold),
          "attention");
    if (fold > 0) {
        TIMED(SSD_K_GEMV_O, gemv_resid_attn(D, c->wo[l], c->f(c->lay.part), fold, x, nullptr, c->stream), "gemv_o");
    } else {
        TIMED(SSD_K_GEMV_O, gemv_resid(D, c->wo[l], D.d, D.dq, c->f(c->lay.att), x, nullptr, c->stream), "gemv_o");
    }
    }
    if (!do_mlp) return SSD_OK;
    TIMED(SSD_K_GEMV_GATEUP, gemv_swiglu(D, c->wg[l], c->wu[l], c->mlp_norm[l], x, c->f(c->lay.act), c->stream),
          "gemv_swiglu");
    TIMED(SSD_K_GEMV_DOWN, gemv_resid(D, c->wd[l], D.d, D.f, c->f(c->lay.act), x, nullptr, c->stream), "gemv_down");
    return SSD_OK;
}

// Single-row forward of the token in tok slot `slot` at position *pos + pos_off; the greedy token goes to
// tok slot `slot_out`, its logits to logits row `lrow`, its max-probability to SM_MAXPROB[lrow].
// sub (may be null): two entries per layer, [2l] != 0 leaves out the attention sub-block, [2l+1] != 0 the MLP sub-block.
int forward_single(ssd_ctx* c, const uint8_t* sub, int slot, int slot_out, int pos_off, int lrow)
{
    const Dims& D = c->D;
    HIPCHK(embed_rows(D, c->w.embed, c->small_i() + SM_TOK + slot, 1, c->f(c->lay.x), c->stream), "embed");
    for (int l = 0; l < D.L; l++) {
        const bool do_attn = !(sub && sub[2 * l]), do_mlp = !(sub && sub[2 * l + 1]);
        if (!do_attn && !do_mlp) continue;
        int rc = layer_single(c, l, pos_off, do_attn, do_mlp);
        if (rc) return rc;
    }
    float* logits = c->f(c->lay.logits) + (size_t)lrow * D.V;
    // LM head with the greedy token and its soft-max probability folded in (block statistics in the attention
    // scratch, which is idle here, then a one-block fold)
    TIMED(SSD_K_GEMV_LMHEAD, gemv_lmhead_argmax(D, c->w.lm_head, c->w.final_norm, c->f(c->lay.x), logits, c->cfg.conf_clamp,
                                                c->f(c->lay.part), c->small_i() + SM_TOK + slot_out,
                                                c->small_f() + SM_MAXPROB + lrow, c->stream), "gemv_lmhead");
    return SSD_OK;
}

// Full-model forward of the M tokens in SM_VTOK (M <= 16, or <= 64 where the wide tiling applies) at positions
// *pos + pos_off + r; taps into tap rows 0..M-1; logits (when want_logits) into logits rows 0..M-1 and greedy tokens
// into SM_TARGET -- for a block of more than 16 rows (a prompt block) only the last row's.
int forward_rows(ssd_ctx* c, int M, int pos_off, int pos_host, bool want_logits, const int32_t* tok_dev = nullptr)
{
    const Dims& D = c->D;
    const Layout& Y = c->lay;
    float* x = c->f(Y.x);
    float* h = c->f(Y.h);
    HIPCHK(embed_rows(D, c->w.embed, tok_dev ? tok_dev : c->small_i() + SM_VTOK, M, x, c->stream), "embed");
    const int tap_ld = D.L * 2 * D.d;
    if (M > 16) {
        // prompt block: the same sequence as the 16-row path below, on 128 x 128 tiles over all rows of the block at
        // once (up to SSD_PREFILL_ROWS), or on 64-row weight tiles (up to 64 rows) where the shape does not fit those.
        // Only the last row of the last block leaves taps (in tap row 0), logits (row 0) and its greedy token
        // (SM_TARGET[0]) behind.
        const bool big = rows_big_supported(D);
        if (big ? M > Y.rows : (!rows_wide_supported(D) || M > 64)) return fail(c, SSD_ECAPACITY, "row block too large for this shape");
        auto gemm = [&](const RowsFused& f) { return big ? rows_big(D, f, c->stream) : rows_wide(D, f, c->stream); };
        uint16_t* hi = c->h16(Y.hi);
        uint16_t* lo = c->h16(Y.lo);
        uint16_t* xh = c->h16(Y.h);
        uint16_t* xl = xh + (size_t)Y.rows * D.d;
        float* ssq = c->f(Y.ssq);
        const int n_ssq = D.d / 64;
        HIPCHK(rows_gain_split(D, x, D.d, c->attn_norm[0], M, D.d, xh, xl, ssq, 64, c->stream), "rows_gain_split");
        for (int l = 0; l < D.L; l++) {
            RowsFused q = {};
            q.w[0] = c->wq[l]; q.w[1] = c->wk[l]; q.w[2] = c->wv[l]; q.n[0] = D.dq; q.n[1] = D.dkv; q.n[2] = D.dkv;
            q.K = D.d; q.bh = xh; q.bl = xl; q.ldb = D.d; q.ssq = ssq; q.n_ssq = n_ssq; q.y = c->f(Y.qkv); q.ldy = D.dq;
            q.M = M; q.mode = 3;
            q.rope = c->f(Y.rope); q.pos_dev = c->pos_dev(); q.pos_off = pos_off; q.kc = c->kcache(l); q.vc = c->vcache(l);
            q.kpart = c->f(Y.part); q.kpart_floats = Y.part_floats;   // the attention scratch is idle outside attention
            TIMED(SSD_K_ROWS_QKV, gemm(q), "wide_qkv");
            TIMED(SSD_K_ATTENTION, attention(D, c->f(Y.qkv), D.dq, c->kcache(l), c->vcache(l), c->pos_dev(), pos_off,
                                             pos_host, M, c->f(Y.part), nullptr, hi, lo, c->stream), "attention");
            RowsFused o = {};
            o.w[0] = c->wo[l]; o.n[0] = D.d; o.K = D.dq; o.bh = hi; o.bl = lo; o.ldb = D.dq; o.y = x; o.ldy = D.d; o.M = M;
            o.mode = 1; o.tap = want_logits ? c->f(Y.taps) + ((size_t)l * 2 + 0) * D.d : nullptr; o.tap_ld = tap_ld; o.tap_only = M;
            o.gain_out = c->mlp_norm[l]; o.oh = xh; o.ol = xl; o.ldo = D.d; o.ssq_out = ssq;
            o.kpart = c->f(Y.part); o.kpart_floats = Y.part_floats;   // attention is done with its scratch
            TIMED(SSD_K_ROWS_O, gemm(o), "wide_o");
            RowsFused gu = {};
            gu.w[0] = c->wg[l]; gu.w[1] = c->wu[l]; gu.n[0] = D.f; gu.n[1] = D.f; gu.K = D.d; gu.bh = xh; gu.bl = xl;
            gu.ldb = D.d; gu.ssq = ssq; gu.n_ssq = n_ssq;
            gu.oh = c->h16(Y.act); gu.ol = c->h16(Y.act) + (size_t)Y.rows * D.f; gu.ldo = D.f; gu.M = M;
            gu.mode = 2;
            gu.kpart = c->f(Y.part); gu.kpart_floats = Y.part_floats;
            TIMED(SSD_K_ROWS_GATEUP, gemm(gu), "wide_gateup");
            RowsFused dn = {};
            dn.w[0] = c->wd[l]; dn.n[0] = D.d; dn.K = D.f; dn.bh = gu.oh; dn.bl = gu.ol; dn.ldb = D.f; dn.y = x; dn.ldy = D.d;
            dn.M = M; dn.mode = 1; dn.tap = want_logits ? c->f(Y.taps) + ((size_t)l * 2 + 1) * D.d : nullptr; dn.tap_ld = tap_ld;
            dn.tap_only = M;
            if (l + 1 < D.L || want_logits) {
                dn.gain_out = l + 1 < D.L ? c->attn_norm[l + 1] : c->w.final_norm;
                dn.oh = xh; dn.ol = xl; dn.ldo = D.d; dn.ssq_out = ssq;
            }
            dn.kpart = c->f(Y.part); dn.kpart_floats = Y.part_floats;
            TIMED(SSD_K_ROWS_DOWN, gemm(dn), "wide_down");
        }
        if (want_logits) {   // last row only, through the 16-row kernel with one row
            const int r = M - 1;
            RowsFused lm = {};
            lm.w[0] = c->w.lm_head; lm.n[0] = D.V; lm.K = D.d; lm.bh = xh + (size_t)r * D.d; lm.bl = xl + (size_t)r * D.d;
            lm.ldb = D.d; lm.ssq = ssq + (size_t)r * n_ssq; lm.n_ssq = n_ssq; lm.y = c->f(Y.logits);
            lm.ldy = D.V; lm.M = 1; lm.mode = 0;
            TIMED(SSD_K_ROWS_LMHEAD, rows_fused(D, lm, c->stream), "rows_lmhead");
            HIPCHK(vocab_reduce(c->f(Y.logits), 1, D.V, c->cfg.conf_clamp, c->cfg.conf_eps,
                                c->small_i() + SM_TARGET, 1, nullptr, nullptr, nullptr, c->stream), "vocab_reduce");
        }
        return SSD_OK;
    }
    if (rows_fused_supported(D)) {
        // 16-bit fast path: activations travel between the GEMMs as hi/lo pairs of the weights' type.  The residual rows exist
        // twice: x (fp32) and xh/xl = split(x * gain of the norm that reads them next) with their per-tile
        // sums of squares in ssq, both left behind by the projection that last updated x.
        uint16_t* hi = c->h16(Y.hi);
        uint16_t* lo = c->h16(Y.lo);
        uint16_t* xh = c->h16(Y.h);
        uint16_t* xl = xh + (size_t)Y.rows * D.d;
        float* ssq = c->f(Y.ssq);
        const int n_ssq = D.d / 16;
        HIPCHK(rows_gain_split(D, x, D.d, c->attn_norm[0], M, D.d, xh, xl, ssq, 16, c->stream), "rows_gain_split");
        for (int l = 0; l < D.L; l++) {
            RowsFused q = {};
            q.w[0] = c->wq[l]; q.w[1] = c->wk[l]; q.w[2] = c->wv[l]; q.n[0] = D.dq; q.n[1] = D.dkv; q.n[2] = D.dkv;
            q.K = D.d; q.bh = xh; q.bl = xl; q.ldb = D.d; q.ssq = ssq; q.n_ssq = n_ssq; q.y = c->f(Y.qkv); q.ldy = D.dq;
            q.M = M; q.mode = 3;
            q.rope = c->f(Y.rope); q.pos_dev = c->pos_dev(); q.pos_off = pos_off; q.kc = c->kcache(l); q.vc = c->vcache(l);
            TIMED(SSD_K_ROWS_QKV, rows_fused(D, q, c->stream), "rows_qkv");
            TIMED(SSD_K_ATTENTION, attention(D, c->f(Y.qkv), D.dq, c->kcache(l), c->vcache(l), c->pos_dev(), pos_off,
                                             pos_host, M, c->f(Y.part), nullptr, hi, lo, c->stream), "attention");
            RowsFused o = {};
            o.w[0] = c->wo[l]; o.n[0] = D.d; o.K = D.dq; o.bh = hi; o.bl = lo; o.ldb = D.dq; o.y = x; o.ldy = D.d; o.M = M;
            o.mode = 1; o.tap = c->f(Y.taps) + ((size_t)l * 2 + 0) * D.d; o.tap_ld = tap_ld;
            o.gain_out = c->mlp_norm[l]; o.oh = xh; o.ol = xl; o.ldo = D.d; o.ssq_out = ssq;
            TIMED(SSD_K_ROWS_O, rows_fused(D, o, c->stream), "rows_o");
            RowsFused gu = {};
            gu.w[0] = c->wg[l]; gu.w[1] = c->wu[l]; gu.n[0] = D.f; gu.n[1] = D.f; gu.K = D.d; gu.bh = xh; gu.bl = xl;
            gu.ldb = D.d; gu.ssq = ssq; gu.n_ssq = n_ssq;
            gu.oh = c->h16(Y.act); gu.ol = c->h16(Y.act) + (size_t)Y.rows * D.f; gu.ldo = D.f; gu.M = M;
            gu.mode = 2;
            TIMED(SSD_K_ROWS_GATEUP, rows_fused(D, gu, c->stream), "rows_gateup");
            RowsFused dn = {};
            dn.w[0] = c->wd[l]; dn.n[0] = D.d; dn.K = D.f; dn.bh = gu.oh; dn.bl = gu.ol; dn.ldb = D.f; dn.y = x; dn.ldy = D.d;
            dn.M = M; dn.mode = 1; dn.tap = c->f(Y.taps) + ((size_t)l * 2 + 1) * D.d; dn.tap_ld = tap_ld;
            if (l + 1 < D.L || want_logits) {
                dn.gain_out = l + 1 < D.L ? c->attn_norm[l + 1] : c->w.final_norm;
                dn.oh = xh; dn.ol = xl; dn.ldo = D.d; dn.ssq_out = ssq;
            }
            TIMED(SSD_K_ROWS_DOWN, rows_fused(D, dn, c->stream), "rows_down");
        }
        if (want_logits) {
            RowsFused lm = {};
            lm.w[0] = c->w.lm_head; lm.n[0] = D.V; lm.K = D.d; lm.bh = xh; lm.bl = xl; lm.ldb = D.d; lm.ssq = ssq;
            lm.n_ssq = n_ssq; lm.y = c->f(Y.logits); lm.ldy = D.V; lm.M = M; lm.mode = 0;
            TIMED(SSD_K_ROWS_LMHEAD, rows_fused(D, lm, c->stream), "rows_lmhead");
            HIPCHK(vocab_reduce(c->f(Y.logits), M, D.V, c->cfg.conf_clamp, c->cfg.conf_eps, c->small_i() + SM_TARGET, 1,
                                nullptr, nullptr, nullptr, c->stream), "vocab_reduce");
        }
        return SSD_OK;
    }
    for (int l = 0; l < D.L; l++) {
        HIPCHK(rmsnorm_rows(x, c->attn_norm[l], M, D.d, D.eps, h, c->stream), "rmsnorm");
        RowsGemm g = {};
        g.w[0] = c->wq[l]; g.w[1] = c->wk[l]; g.w[2] = c->wv[l];
        g.n[0] = D.dq; g.n[1] = D.dkv; g.n[2] = D.dkv;
        g.K = D.d; g.x = h; g.y = c->f(Y.qkv); g.ldy = D.dq + 2 * D.dkv; g.M = M; g.mode = 0;
        TIMED(SSD_K_ROWS_QKV, gemm_rows(D, g, c->stream), "gemm_qkv");
        HIPCHK(rope_kv_rows(D, c->f(Y.qkv), c->f(Y.rope), c->pos_dev(), pos_off, M, c->kcache(l), c->vcache(l),
                            c->stream), "rope_kv");
        TIMED(SSD_K_ATTENTION, attention(D, c->f(Y.qkv), D.dq + 2 * D.dkv, c->kcache(l), c->vcache(l), c->pos_dev(),
                                         pos_off, pos_host, M, c->f(Y.part), c->f(Y.att), nullptr, nullptr, c->stream), "attention");
        RowsGemm o = {};
        o.w[0] = c->wo[l]; o.n[0] = D.d; o.K = D.dq; o.x = c->f(Y.att); o.y = x; o.ldy = D.d; o.M = M; o.mode = 1;
        o.tap = c->f(Y.taps) + ((size_t)l * 2 + 0) * D.d; o.tap_ld = tap_ld;
        TIMED(SSD_K_ROWS_O, gemm_rows(D, o, c->stream), "gemm_o");
        HIPCHK(rmsnorm_rows(x, c->mlp_norm[l], M, D.d, D.eps, h, c->stream), "rmsnorm");
        RowsGemm gu = {};
        gu.w[0] = c->wg[l]; gu.w[1] = c->wu[l]; gu.n[0] = D.f; gu.n[1] = D.f; gu.K = D.d; gu.x = h;
        gu.y = c->f(Y.act); gu.ldy = D.f; gu.M = M; gu.mode = 2;
        TIMED(SSD_K_ROWS_GATEUP, gemm_rows(D, gu, c->stream), "gemm_gateup");
        RowsGemm dn = {};
        dn.w[0] = c->wd[l]; dn.n[0] = D.d; dn.K = D.f; dn.x = c->f(Y.act); dn.y = x; dn.ldy = D.d; dn.M = M; dn.mode = 1;
        dn.tap = c->f(Y.taps) + ((size_t)l * 2 + 1) * D.d; dn.tap_ld = tap_ld;
        TIMED(SSD_K_ROWS_DOWN, gemm_rows(D, dn, c->stream), "gemm_down");
    }
    if (want_logits) {
        HIPCHK(rmsnorm_rows(x, c->w.final_norm, M, D.d, D.eps, h, c->stream), "rmsnorm");
        RowsGemm lm = {};
        lm.w[0] = c->w.lm_head; lm.n[0] = D.V; lm.K = D.d; lm.x = h; lm.y = c->f(Y.logits); lm.ldy = D.V; lm.M = M;
        lm.mode = 0;
        TIMED(SSD_K_ROWS_LMHEAD, gemm_rows(D, lm, c->stream), "gemm_lmhead");
        HIPCHK(vocab_reduce(c->f(Y.logits), M, D.V, c->cfg.conf_clamp, c->cfg.conf_eps, c->small_i() + SM_TARGET, 1,
                            nullptr, nullptr, nullptr, c->stream), "vocab_reduce");
    }
    return SSD_OK;
}

// Runs a launch sequence.  The first time a key is seen the sequence runs kernel by kernel; the
// second time it is captured into a HIP graph, and from then on the graph is replayed (one
// submission instead of hundreds of launches).  Everything position-dependent is read from
// device memory by the kernels, so a graph stays valid as the sequence grows; what is baked into
// it (skip mask, k, attention split counts) is part of the key.
template <typename F>
int run_sequence(ssd_ctx* c, const std::string& key, F&& body)
{
    if (!c->use_graphs || c->prof_kid >= 0 || c->stream == nullptr) return body();
    auto it = c->graphs.find(key);
    if (it == c->graphs.end()) {
        if (c->graphs.size() >= 256) {  // masks change during the search: keep the cache bounded
            for (auto& e : c->graphs)
                if (e.second) (void)hipGraphExecDestroy(e.second);
            c->graphs.clear();
        }
        c->graphs[key] = nullptr;
        return body();
    }
    if (!it->second) {
        HIPCHK(hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed), "begin capture");
        int rc = body();
        hipGraph_t g = nullptr;
        hipError_t e = hipStreamEndCapture(c->stream, &g);
        if (rc != SSD_OK || e != hipSuccess || !g) {
            if (g) (void)hipGraphDestroy(g);
            c->graphs.erase(it);
            return rc != SSD_OK ? rc : hip_fail(c, e, "end capture");
        }
        hipGraphExec_t exec = nullptr;
        e = hipGraphInstantiate(&exec, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (e != hipSuccess) { c->graphs.erase(it); return hip_fail(c, e, "graph instantiate"); }
        it->second = exec;
    }
    HIPCHK(hipGraphLaunch(it->second, c->stream), "graph launch");
    return SSD_OK;
}

int readback(ssd_ctx* c, const void* dev, size_t bytes, void* host)
{
    HIPCHK(hipMemcpyAsync(c->pinned, dev, bytes, hipMemcpyDeviceToHost, c->stream), "readback copy");
    HIPCHK(hipStreamSynchronize(c->stream), "readback sync");
    memcpy(host, c->pinned, bytes);
    return SSD_OK;
}


// Device buffers one confidence pass works in: hi/lo pairs of the normalised tap rows (16-bit weights), the normalised
// rows themselves (fp32 weights), their logits, and 3 result values per row; `batch` tap rows go through per pass.
struct ConfScratch {
    uint16_t* hi; uint16_t* lo; float* tapn; float* logits; float* res; int batch;
    bool one_gemm;   // the context-window pass: a batch of more than 64 rows goes through the 128 x 128-tile GEMM in
                     // one launch (the per-layer passes keep 64-row launches whatever their batch, so that the two
                     // entry points for them run the same kernels on the same tiles)
};

// Enqueues the confidence (Eq. 1-4) of nb tap rows [nb][d] (nb <= sc.batch): final norm, LM head, vocabulary
// reduction; one value per row to conf_dev, and to maxprob_dev / argmax_dev when given (device pointers).
int conf_batch(ssd_ctx* c, const ConfScratch& sc, const float* taps, int nb, float* conf_dev, float* maxprob_dev,
               int32_t* argmax_dev)
{
    const Dims& D = c->D;
    if (rows_fused_supported(D)) {
        HIPCHK(rows_prep(D, taps, D.d, c->w.final_norm, nb, D.d, D.eps, sc.hi, sc.lo, c->stream), "rows_prep taps");
        if (sc.one_gemm && nb > 64 && rows_big_supported(D)) {   // a real GEMM: all rows against the LM head in one launch
            RowsFused lm = {};
            lm.w[0] = c->w.lm_head; lm.n[0] = D.V; lm.K = D.d; lm.bh = sc.hi; lm.bl = sc.lo; lm.ldb = D.d;
            lm.y = sc.logits; lm.ldy = D.V; lm.M = nb; lm.mode = 0;
            TIMED(SSD_K_ROWS_LMHEAD, rows_big(D, lm, c->stream), "rows conf lmhead");
        } else if (rows_many_supported(D, D.V, D.d)) {
            for (int b = 0; b < nb; b += 64) {   // the LM head is streamed once per 64 tap rows
                TIMED(SSD_K_ROWS_LMHEAD, rows_many(D, c->w.lm_head, D.V, D.d, sc.hi + (size_t)b * D.d, sc.lo + (size_t)b * D.d,
                                                   D.d, nb - b < 64 ? nb - b : 64, sc.logits + (size_t)b * D.V, D.V, c->stream),
                      "rows conf lmhead");
            }
        } else {
            for (int b = 0; b < nb; b += 16) {
                RowsFused lm = {};
                lm.w[0] = c->w.lm_head; lm.n[0] = D.V; lm.K = D.d; lm.bh = sc.hi + (size_t)b * D.d;
                lm.bl = sc.lo + (size_t)b * D.d; lm.ldb = D.d; lm.y = sc.logits + (size_t)b * D.V; lm.ldy = D.V;
                lm.M = nb - b < 16 ? nb - b : 16; lm.mode = 0;
                TIMED(SSD_K_ROWS_LMHEAD, rows_fused(D, lm, c->stream), "rows conf lmhead");
            }
        }
    } else {
        HIPCHK(rmsnorm_rows(taps, c->w.final_norm, nb, D.d, D.eps, sc.tapn, c->stream), "rmsnorm taps");
        for (int b = 0; b < nb; b += 16) {
            RowsGemm lm = {};
            lm.w[0] = c->w.lm_head; lm.n[0] = D.V; lm.K = D.d; lm.x = sc.tapn + (size_t)b * D.d;
            lm.y = sc.logits + (size_t)b * D.V; lm.ldy = D.V; lm.M = nb - b < 16 ? nb - b : 16; lm.mode = 0;
            TIMED(SSD_K_ROWS_LMHEAD, gemm_rows(D, lm, c->stream), "gemm conf lmhead");
        }
    }
    HIPCHK(vocab_reduce(sc.logits, nb, D.V, c->cfg.conf_clamp, c->cfg.conf_eps, nullptr, 1, argmax_dev, maxprob_dev, conf_dev,
                        c->stream), "vocab_reduce conf");
    return SSD_OK;
}

// Confidence (Eq. 1-4) of all 2L tap rows of positions [row_begin, row_begin + n_rows) of the tap buffer, `sc.batch`
// tap rows at a time; results to the host arrays.  timed: launches of the LM head may be bracketed by profiling events.
int confidence_rows(ssd_ctx* c, const ConfScratch& sc, int row_begin, int n_rows, float* conf_out, float* tap_conf_out,
                    float* tap_maxprob_out, int32_t* tap_argmax_out, bool timed)
{
    const Dims& D = c->D;
    const Layout& Y = c->lay;
    const int R = 2 * D.L;
    const int saved_kid = c->prof_kid;
    if (!timed) c->prof_kid = -1;           // (event creation allocates)
    struct Restore { ssd_ctx* c; int kid; ~Restore() { c->prof_kid = kid; } } restore{c, saved_kid};
    float hb[3 * 2 * SSD_MAX_LAYERS];
    for (int r = 0; r < n_rows; r++) {
        const float* taps_row = c->f(Y.taps) + (size_t)(c->tap_row0 + row_begin + r) * R * D.d;  // [L][2][d]
        for (int b0 = 0; b0 < R; b0 += sc.batch) {
            const int nb = R - b0 < sc.batch ? R - b0 : sc.batch;
            int rc = conf_batch(c, sc, taps_row + (size_t)b0 * D.d, nb, sc.res, sc.res + nb,
                                reinterpret_cast<int32_t*>(sc.res + 2 * nb));
            if (rc) return rc;
            float tmp[3 * 64 > 3 * 2 * SSD_MAX_LAYERS ? 3 * 64 : 3 * 2 * SSD_MAX_LAYERS];
            rc = readback(c, sc.res, sizeof(float) * 3 * nb, tmp);
            if (rc) return rc;
            for (int i = 0; i < nb; i++) {   // regroup as [R] conf, [R] maxprob, [R] argmax
                hb[b0 + i] = tmp[i]; hb[R + b0 + i] = tmp[nb + i]; hb[2 * R + b0 + i] = tmp[2 * nb + i];
            }
        }
        for (int l = 0; l < D.L; l++) {
            float ca = hb[l * 2], cb = hb[l * 2 + 1];
            conf_out[(size_t)r * D.L + l] = c->cfg.conf_taps == 2 ? 0.5f * (ca + cb) : cb;
            for (int t = 0; t < 2; t++) {
                size_t o = ((size_t)r * D.L + l) * 2 + t;
                if (tap_conf_out) tap_conf_out[o] = hb[l * 2 + t];
                if (tap_maxprob_out) tap_maxprob_out[o] = hb[R + l * 2 + t];
                if (tap_argmax_out) memcpy(&tap_argmax_out[o], &hb[2 * R + l * 2 + t], 4);
            }
        }
    }
    c->st.confidence_rows += (int64_t)n_rows * R;
    return SSD_OK;
}

// Context window (Section 4.1.1): the taps of tap-buffer rows [first, first + n) -- positions the full model has just
// processed with committed input tokens -- enter the device ring of the last conf_window positions.
int ring_push(ssd_ctx* c, int first, int n)
{
    const int Wn = c->cfg.conf_window;
    if (Wn == 0 || n <= 0) return SSD_OK;
    const size_t row = (size_t)2 * c->D.L * c->D.d;     // floats per position
    if (n > Wn) { first += n - Wn; c->ring_count += n - Wn; n = Wn; }   // only the last Wn positions can survive
    while (n > 0) {
        const int slot = (int)(c->ring_count % Wn);
        const int run = n < Wn - slot ? n : Wn - slot;  // contiguous slots up to the end of the ring
        HIPCHK(copy_f32(c->f(c->lay.taps) + (size_t)(c->tap_row0 + first) * row, c->f(c->lay.ring) + (size_t)slot * row,
                        (size_t)run * row, c->stream), "ring push");
        c->ring_count += run; first += run; n -= run;
    }
    return SSD_OK;
}

}  // namespace

extern "C" {

int ssd_create(const ssd_config* cfg, void* hip_stream, ssd_ctx** out)
{
    if (!out) return SSD_EINVAL;
    *out = nullptr;
    if (!valid_cfg(cfg)) return SSD_EINVAL;
    ssd_ctx* c = new ssd_ctx();
    c->cfg = *cfg;
    c->D = make_dims(*cfg);
    c->D.opt = &c->opts;
    c->lay = make_layout(*cfg);
    c->stream = (hipStream_t)hip_stream;
    c->state = ST_CREATED;
    c->ws = nullptr; c->ws_bytes = 0; c->have_w = false;
    c->n = 0; c->k_pending = 0; c->tap_rows = 0; c->tap_row0 = 0; c->logit_rows = 0; c->ring_count = 0; c->pinned = nullptr; c->device = -1; c->static_scratch = nullptr;
    memset(&c->st, 0, sizeof(c->st));
    memset(&c->w, 0, sizeof(c->w));
    c->prof_kid = -1; c->prof_used = 0;
    c->use_graphs = true;
    *out = c;
    return SSD_OK;
}

size_t ssd_workspace_bytes(const ssd_config* cfg)
{
    if (!valid_cfg(cfg)) return 0;
    return make_layout(*cfg).total;
}

int ssd_set_workspace(ssd_ctx* c, void* dev, size_t bytes)
{
    if (!c) return SSD_EINVAL;
    if (!dev || bytes < c->lay.total) return fail(c, SSD_ENOMEM, "workspace missing or smaller than ssd_workspace_bytes");
    if (reinterpret_cast<uintptr_t>(dev) % ALIGN) return fail(c, SSD_EINVAL, "workspace must be 256-byte aligned");
    if (c->state != ST_CREATED && c->state != ST_READY) return fail(c, SSD_ESTATE, "workspace can only be set before prefill");
    // rotary table in double precision on the host: cos/sin(p * base^(-2i/hd))
    const int half = c->D.hd / 2;
    std::vector<float> tab((size_t)c->D.max_seq * half * 2);
    for (int p = 0; p < c->D.max_seq; p++)
        for (int i = 0; i < half; i++) {
            double ang = (double)p * std::pow((double)c->cfg.rope_base, -2.0 * (double)i / (double)c->D.hd);
            tab[((size_t)p * half + i) * 2 + 0] = (float)std::cos(ang);
            tab[((size_t)p * half + i) * 2 + 1] = (float)std::sin(ang);
        }
    if (!c->pinned) HIPCHK(hipHostMalloc((void**)&c->pinned, 64 * 1024, hipHostMallocDefault), "hipHostMalloc");
    HIPCHK(hipGetDevice(&c->device), "hipGetDevice");
    HIPCHK(static_scratch_for_device(c->device, &c->static_scratch), "static scratch address");
    c->ws = static_cast<char*>(dev);
    c->ws_bytes = bytes;
    HIPCHK(hipMemcpyAsync(c->ws + c->lay.rope, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice, c->stream),
           "rope upload");
    HIPCHK(hipMemsetAsync(c->ws + c->lay.small, 0, 4096, c->stream), "state clear");
    HIPCHK(hipStreamSynchronize(c->stream), "workspace sync");  // tab goes out of scope
    if (c->have_w) c->state = ST_READY;
    return SSD_OK;
}

int ssd_load_weights(ssd_ctx* c, const ssd_weights* w)
{
    if (!c || !w) return SSD_EINVAL;
    if (c->state != ST_CREATED && c->state != ST_READY) return fail(c, SSD_ESTATE, "weights can only be loaded before prefill");
    if (!w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
        !w->mlp_norm || !w->wg || !w->wu || !w->wd)
        return fail(c, SSD_EINVAL, "null weight pointer");
    const int L = c->D.L;
    for (int l = 0; l < L; l++)
        if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->mlp_norm[l] || !w->wg[l] ||
            !w->wu[l] || !w->wd[l])
            return fail(c, SSD_EINVAL, "null per-layer weight pointer");
    auto chk = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
    bool ok = chk(w->embed) && chk(w->lm_head) && chk(w->final_norm);
    for (int l = 0; l < L && ok; l++)
        ok = chk(w->attn_norm[l]) && chk(w->wq[l]) && chk(w->wk[l]) && chk(w->wv[l]) && chk(w->wo[l]) &&
             chk(w->mlp_norm[l]) && chk(w->wg[l]) && chk(w->wu[l]) && chk(w->wd[l]);
    if (!ok) return fail(c, SSD_EINVAL, "weight pointers must be 16-byte aligned");
    c->w = *w;
    c->attn_norm.assign(w->attn_norm, w->attn_norm + L);
    c->mlp_norm.assign(w->mlp_norm, w->mlp_norm + L);
    c->wq.assign(w->wq, w->wq + L); c->wk.assign(w->wk, w->wk + L); c->wv.assign(w->wv, w->wv + L);
    c->wo.assign(w->wo, w->wo + L); c->wg.assign(w->wg, w->wg + L); c->wu.assign(w->wu, w->wu + L);
    c->wd.assign(w->wd, w->wd + L);
    c->have_w = true;
    if (c->ws) c->state = ST_READY;
    return SSD_OK;
}

int ssd_reset(ssd_ctx* c)
{
    if (!c) return SSD_EINVAL;
    if (c->state == ST_CREATED) return fail(c, SSD_ESTATE, "nothing to reset");
    c->state = ST_READY;
    c->n = 0; c->k_pending = 0; c->tap_rows = 0; c->logit_rows = 0; c->ring_count = 0;
    memset(&c->st, 0, sizeof(c->st));
    return SSD_OK;
}

void ssd_destroy(ssd_ctx* c)
{
    if (!c) return;
    if (c->pinned) (void)hipHostFree(c->pinned);
    for (auto& e : c->prof_ev) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
    for (auto& e : c->graphs)
        if (e.second) (void)hipGraphExecDestroy(e.second);
    delete c;
}

const char* ssd_last_error(const ssd_ctx* c) { return c ? c->err.c_str() : "null context"; }

int ssd_get_stats(const ssd_ctx* c, ssd_stats* out)
{
    if (!c || !out) return SSD_EINVAL;
    *out = c->st;
    out->n_tokens = c->n;
    out->state = (int32_t)c->state;
    return SSD_OK;
}

int ssd_prefill(ssd_ctx* c, const int32_t* tokens, int n, int32_t* first_token_out)
{
    if (!c || !tokens || !first_token_out || n < 1) return c ? fail(c, SSD_EINVAL, "prefill: bad argument") : SSD_EINVAL;
    if (c->state != ST_READY) return fail(c, SSD_ESTATE, "prefill needs workspace + weights and an empty sequence");
    if (n + 1 > c->D.max_seq) return fail(c, SSD_ECAPACITY, "prompt does not fit max_seq");
    for (int i = 0; i < n; i++)
        if (tokens[i] < 0 || tokens[i] >= c->D.V) return fail(c, SSD_EINVAL, "prompt token id out of range");
    HIPCHK(set_state(c->small_i() + SM_TOK, 0, c->pos_dev(), 0, c->stream), "set_state");
    int last_M = 0;
    const int block = c->lay.prefill_rows;
    int32_t* vtok = reinterpret_cast<int32_t*>(c->ws + c->lay.vtok);
    for (int p0 = 0; p0 < n; p0 += block) {
        int M = n - p0 < block ? n - p0 : block;
        for (int r0 = 0; r0 < M; r0 += 64) {   // token ids travel as kernel arguments, 64 at a time
            TokArg t = {};
            const int nr = M - r0 < 64 ? M - r0 : 64;
            for (int r = 0; r < nr; r++) t.t[r] = tokens[p0 + r0 + r];
            HIPCHK(set_tokens(t, nr, nullptr, vtok + r0, c->stream), "set_tokens");
        }
        bool last = p0 + M == n;
        int rc = forward_rows(c, M, p0, 0, last, vtok);
        if (rc) return rc;
        last_M = M;
    }
    // a block of more than 16 rows leaves its last row's results in row 0, a shorter one in the row itself
    const int res_row = last_M > 16 ? 0 : last_M - 1;
    // pending token = greedy token after the last prompt row; n_cached positions = n
    HIPCHK(advance_state(c->pos_dev(), n, c->small_i() + SM_TOK, c->small_i() + SM_TARGET + res_row, c->stream),
           "advance_state");
    int rc = readback(c, c->small_i() + SM_TARGET + res_row, sizeof(int32_t), first_token_out);
    if (rc) return rc;
    c->n = n + 1;
    c->state = ST_IDLE;
    c->tap_rows = 1; c->tap_row0 = res_row;
    c->logit_rows = 1;
    c->ring_count = 0;
    rc = ring_push(c, 0, 1);    // the last prompt position opens the context window
    if (rc) return rc;
    // logits of the last row sit at row res_row; move them to row 0 so ssd_copy_logits sees one row
    if (res_row > 0) {
        HIPCHK(copy_f32(c->f(c->lay.logits) + (size_t)res_row * c->D.V, c->f(c->lay.logits), c->D.V, c->stream),
               "logits move");
    }
    c->st.committed = 1;
    return SSD_OK;
}

int ssd_decode(ssd_ctx* c, int32_t* token_out)
{
    if (!c || !token_out) return c ? fail(c, SSD_EINVAL, "decode: bad argument") : SSD_EINVAL;
    if (c->state != ST_IDLE) return fail(c, SSD_ESTATE, "decode needs a prefilled sequence with no draft in flight");
    if (c->n + 1 > c->D.max_seq) return fail(c, SSD_ECAPACITY, "sequence would exceed max_seq");
    // pending token sits in tok slot 0; its successor is written to slot 1, then promoted
    std::string key = "D|" + std::to_string(attention_splits(c->D, c->n, 1));
    int rc = run_sequence(c, key, [&]() {
        int r = forward_single(c, nullptr, 0, 1, 0, 0);
        if (r) return r;
        HIPCHK(advance_state(c->pos_dev(), 1, c->small_i() + SM_TOK, c->small_i() + SM_TOK + 1, c->stream), "advance_state");
        return (int)SSD_OK;
    });
    if (rc) return rc;
    rc = readback(c, c->small_i() + SM_TOK + 1, sizeof(int32_t), token_out);
    if (rc) return rc;
    c->n += 1;
    c->logit_rows = 1;
    c->tap_rows = 0;
    c->st.decode_steps++; c->st.committed++;
    return SSD_OK;
}

// Common body of the two fixed-length draft calls; sub has two entries per layer.
static int draft_fixed(ssd_ctx* c, const std::vector<uint8_t>& sub, int k, int32_t* draft_out, float* draft_maxprob_out)
{
    if (k < 1) return fail(c, SSD_EINVAL, "k must be at least 1");
    if (c->state != ST_IDLE) return fail(c, SSD_ESTATE, "draft_step needs a prefilled sequence with no draft in flight");
    if (k > c->cfg.max_k) return fail(c, SSD_ECAPACITY, "k exceeds max_k");
    if (c->n + k > c->D.max_seq) return fail(c, SSD_ECAPACITY, "draft + verification would exceed max_seq");
    std::string key = "S|" + std::to_string(k) + "|" + std::string(sub.begin(), sub.end()) + "|";
    for (int i = 0; i < k; i++) key += std::to_string(attention_splits(c->D, c->n + i, 1)) + ",";
    int rc = run_sequence(c, key, [&]() {
        for (int i = 0; i < k; i++) {
            int r = forward_single(c, sub.data(), i, i + 1, i, i);
            if (r) return r;
        }
        return (int)SSD_OK;
    });
    if (rc) return rc;
    rc = readback(c, c->small_i() + SM_TOK + 1, sizeof(int32_t) * k, draft_out);
    if (rc) return rc;
    if (draft_maxprob_out) {
        rc = readback(c, c->small_f() + SM_MAXPROB, sizeof(float) * k, draft_maxprob_out);
        if (rc) return rc;
    }
    c->state = ST_DRAFTED;
    c->k_pending = k;
    c->logit_rows = k;
    c->tap_rows = 0;
    c->st.draft_steps += k;
    return SSD_OK;
}

// whole-layer mask [L] -> sub-block mask [2L] with 0 / 1 entries
static std::vector<uint8_t> expand_mask(const uint8_t* skip_mask, int L)
{
    std::vector<uint8_t> sub((size_t)2 * L);
    for (int l = 0; l < L; l++) sub[2 * l] = sub[2 * l + 1] = skip_mask[l] ? 1 : 0;
    return sub;
}

int ssd_draft_step(ssd_ctx* c, const uint8_t* skip_mask, int k, int32_t* draft_out, float* draft_maxprob_out)
{
    if (!c || !skip_mask || !draft_out) return c ? fail(c, SSD_EINVAL, "draft_step: bad argument") : SSD_EINVAL;
    return draft_fixed(c, expand_mask(skip_mask, c->D.L), k, draft_out, draft_maxprob_out);
}

int ssd_draft_step_sub(ssd_ctx* c, const uint8_t* sub_mask, int k, int32_t* draft_out, float* draft_maxprob_out)
{
    if (!c || !sub_mask || !draft_out) return c ? fail(c, SSD_EINVAL, "draft_step_sub: bad argument") : SSD_EINVAL;
    std::vector<uint8_t> sub((size_t)2 * c->D.L);
    for (size_t i = 0; i < sub.size(); i++) sub[i] = sub_mask[i] ? 1 : 0;
    return draft_fixed(c, sub, k, draft_out, draft_maxprob_out);
}

int ssd_draft_adaptive(ssd_ctx* c, const uint8_t* skip_mask, int k_max, float gamma, int32_t* draft_out,
                       float* draft_maxprob_out, int32_t* k_out)
{
    if (!c || !skip_mask || !draft_out || !k_out) return c ? fail(c, SSD_EINVAL, "draft_adaptive: bad argument") : SSD_EINVAL;
    if (k_max < 1) return fail(c, SSD_EINVAL, "k_max must be at least 1");
    if (gamma != gamma) return fail(c, SSD_EINVAL, "gamma is NaN");
    if (c->state != ST_IDLE) return fail(c, SSD_ESTATE, "draft_adaptive needs a prefilled sequence with no draft in flight");
    if (k_max > c->cfg.max_k) return fail(c, SSD_ECAPACITY, "k_max exceeds max_k");
    if (c->n + k_max > c->D.max_seq) return fail(c, SSD_ECAPACITY, "draft + verification would exceed max_seq");
    const std::vector<uint8_t> sub = expand_mask(skip_mask, c->D.L);
    const std::string mask_key(sub.begin(), sub.end());
    int k = 0;
    while (k < k_max) {
        // one draft step per submission: the host reads the step's max-probability before deciding on the next
        const int i = k;
        std::string key = "A|" + std::to_string(i) + "|" + mask_key + "|" + std::to_string(attention_splits(c->D, c->n + i, 1));
        int rc = run_sequence(c, key, [&]() { return forward_single(c, sub.data(), i, i + 1, i, i); });
        if (rc) return rc;
        float p = 0.f;
        rc = readback(c, c->small_f() + SM_MAXPROB + i, sizeof(float), &p);
        if (rc) return rc;
        k++;
        if (draft_maxprob_out) draft_maxprob_out[i] = p;
        if (p < gamma) break;
    }
    int rc = readback(c, c->small_i() + SM_TOK + 1, sizeof(int32_t) * k, draft_out);
    if (rc) return rc;
    *k_out = k;
    c->state = ST_DRAFTED;
    c->k_pending = k;
    c->logit_rows = k;
    c->tap_rows = 0;
    c->st.draft_steps += k;
    return SSD_OK;
}

int ssd_verify(ssd_ctx* c, const int32_t* draft, int k, int32_t* target_out)
{
    if (!c || !draft || !target_out) return c ? fail(c, SSD_EINVAL, "verify: bad argument") : SSD_EINVAL;
    if (c->state != ST_DRAFTED) return fail(c, SSD_ESTATE, "verify must follow draft_step");
    if (k != c->k_pending) return fail(c, SSD_EINVAL, "verify: k differs from the draft's");
    for (int i = 0; i < k; i++)
        if (draft[i] < 0 || draft[i] >= c->D.V) return fail(c, SSD_EINVAL, "draft token id out of range");
    TokArg t = {};
    for (int i = 0; i < k; i++) t.t[i + 1] = draft[i];
    HIPCHK(set_tokens(t, k + 1, c->small_i() + SM_TOK, c->small_i() + SM_VTOK, c->stream), "set_tokens");
    std::string key = "V|" + std::to_string(k) + "|" + std::to_string(attention_splits(c->D, c->n + k, k + 1));
    int rc = run_sequence(c, key, [&]() { return forward_rows(c, k + 1, 0, c->n - 1, true); });
    if (rc) return rc;
    rc = readback(c, c->small_i() + SM_TARGET, sizeof(int32_t) * (k + 1), target_out);
    if (rc) return rc;
    c->state = ST_VERIFIED;
    c->tap_rows = k + 1; c->tap_row0 = 0;
    c->logit_rows = k + 1;
    c->st.verify_rows += k + 1;
    return SSD_OK;
}

int ssd_accept(ssd_ctx* c, const int32_t* draft, const int32_t* target, int k, int32_t* n_accepted_out,
               int32_t* next_token_out)
{
    if (!c || !draft || !target || !n_accepted_out || !next_token_out)
        return c ? fail(c, SSD_EINVAL, "accept: bad argument") : SSD_EINVAL;
    if (c->state != ST_VERIFIED) return fail(c, SSD_ESTATE, "accept must follow verify");
    if (k != c->k_pending) return fail(c, SSD_EINVAL, "accept: k differs from the draft's");
    for (int i = 0; i <= k; i++)
        if (target[i] < 0 || target[i] >= c->D.V) return fail(c, SSD_EINVAL, "target token id out of range");
    // Both token arrays are on the host already: the prefix match is taken here and the device-side state (pending
    // token, position) is updated by an enqueued kernel -- no read-back, no synchronisation in this call.
    int32_t res[2];
    res[0] = 0;
    while (res[0] < k && draft[res[0]] == target[res[0]]) res[0]++;
    res[1] = target[res[0]];
    HIPCHK(set_state(c->small_i() + SM_TOK, res[1], c->pos_dev(), c->n - 1 + res[0] + 1, c->stream), "accept state update");
    {   // verify rows 0..a were fed committed tokens: their taps enter the context window
        int rc = ring_push(c, 0, res[0] + 1);
        if (rc) return rc;
    }
    *n_accepted_out = res[0];
    *next_token_out = res[1];
    c->n += res[0] + 1;
    c->state = ST_IDLE;
    c->k_pending = 0;
    c->st.cycles++; c->st.drafted += k; c->st.accepted += res[0]; c->st.committed += res[0] + 1;
    return SSD_OK;
}

int ssd_force_commit(ssd_ctx* c, const int32_t* draft, int k, int n_accepted, int32_t next_token)
{
    if (!c || !draft) return c ? fail(c, SSD_EINVAL, "force_commit: bad argument") : SSD_EINVAL;
    if (c->state != ST_VERIFIED) return fail(c, SSD_ESTATE, "force_commit must follow verify");
    if (k != c->k_pending || n_accepted < 0 || n_accepted > k || next_token < 0 || next_token >= c->D.V)
        return fail(c, SSD_EINVAL, "force_commit: bad argument");
    HIPCHK(set_state(c->small_i() + SM_TOK, next_token, c->pos_dev(), c->n - 1 + n_accepted + 1, c->stream), "set_state");
    {
        int rc = ring_push(c, 0, n_accepted + 1);
        if (rc) return rc;
    }
    HIPCHK(hipStreamSynchronize(c->stream), "sync");
    c->n += n_accepted + 1;
    c->state = ST_IDLE;
    c->k_pending = 0;
    c->st.cycles++; c->st.drafted += k; c->st.accepted += n_accepted; c->st.committed += n_accepted + 1;
    return SSD_OK;
}

int ssd_copy_logits(ssd_ctx* c, int row_begin, int n_rows, float* logits_out)
{
    if (!c || !logits_out || row_begin < 0 || n_rows < 1) return c ? fail(c, SSD_EINVAL, "copy_logits: bad argument") : SSD_EINVAL;
    if (c->state < ST_IDLE) return fail(c, SSD_ESTATE, "no logits yet");
    if (row_begin + n_rows > c->logit_rows) return fail(c, SSD_EINVAL, "copy_logits: rows out of range");
    HIPCHK(hipMemcpyAsync(logits_out, c->f(c->lay.logits) + (size_t)row_begin * c->D.V,
                          (size_t)n_rows * c->D.V * sizeof(float), hipMemcpyDeviceToHost, c->stream), "logits copy");
    HIPCHK(hipStreamSynchronize(c->stream), "sync");
    return SSD_OK;
}

int ssd_layer_confidence(ssd_ctx* c, int row_begin, int n_rows, float* conf_out, float* tap_conf_out,
                         float* tap_maxprob_out, int32_t* tap_argmax_out)
{
    if (!c || !conf_out || row_begin < 0 || n_rows < 1) return c ? fail(c, SSD_EINVAL, "layer_confidence: bad argument") : SSD_EINVAL;
    if (c->state < ST_IDLE || c->tap_rows == 0) return fail(c, SSD_ESTATE, "no hidden-state taps: call after prefill or verify");
    if (row_begin + n_rows > c->tap_rows) return fail(c, SSD_EINVAL, "layer_confidence: rows out of range");
    const Layout& Y = c->lay;
    static_assert(SM_CONF + 3 * 2 * SSD_MAX_LAYERS <= SM_VTOK, "confidence results of 2 x SSD_MAX_LAYERS rows must end before the token slots");
    ConfScratch sc;
    sc.hi = c->h16(Y.hi); sc.lo = c->h16(Y.lo); sc.tapn = c->f(Y.tapn); sc.logits = c->f(Y.logits);
    sc.res = c->small_f() + SM_CONF; sc.batch = 2 * c->D.L;     // all tap rows of a position in one pass
    sc.one_gemm = false;
    int rc = confidence_rows(c, sc, row_begin, n_rows, conf_out, tap_conf_out, tap_maxprob_out, tap_argmax_out, true);
    if (rc) return rc;
    c->logit_rows = 0;  // the logits buffer was reused
    return SSD_OK;
}

int ssd_layer_confidence_static(ssd_ctx* c, int row_begin, int n_rows, float* conf_out, float* tap_conf_out,
                                float* tap_maxprob_out, int32_t* tap_argmax_out)
{
    if (!c || !conf_out || row_begin < 0 || n_rows < 1)
        return c ? fail(c, SSD_EINVAL, "layer_confidence_static: bad argument") : SSD_EINVAL;
    if (c->state < ST_IDLE || c->tap_rows == 0) return fail(c, SSD_ESTATE, "no hidden-state taps: call after prefill or verify");
    if (row_begin + n_rows > c->tap_rows) return fail(c, SSD_EINVAL, "layer_confidence_static: rows out of range");
    if (!c->static_scratch) return fail(c, SSD_ESTATE, "the device's static scratch was not resolved (set_workspace failed?)");
    int dev = -1;
    HIPCHK(hipGetDevice(&dev), "hipGetDevice");
    if (dev != c->device) return fail(c, SSD_EINVAL, "layer_confidence_static: the context's device is not current");
    // carve the device's static array: hi, lo, normalised rows (fp32 path), logits, results for one batch of rows
    const Dims& D = c->D;
    const int R = 2 * D.L, B = R < 64 ? R : 64;
    size_t o = 0;
    ConfScratch sc;
    char* base = static_cast<char*>(c->static_scratch);
    sc.hi = reinterpret_cast<uint16_t*>(base + o);   o += align_up((size_t)B * D.d * 2);
    sc.lo = reinterpret_cast<uint16_t*>(base + o);   o += align_up((size_t)B * D.d * 2);
    sc.tapn = reinterpret_cast<float*>(base + o);    o += align_up(rows_fused_supported(D) ? 0 : (size_t)B * D.d * 4);
    sc.logits = reinterpret_cast<float*>(base + o);  o += align_up((size_t)B * D.V * 4);
    sc.res = reinterpret_cast<float*>(base + o);     o += align_up((size_t)3 * B * 4);
    sc.batch = B; sc.one_gemm = false;
    if (o > static_scratch_bytes())
        return fail(c, SSD_ECAPACITY, "layer_confidence_static: 64 rows of this vocabulary / width exceed SSD_STATIC_SCRATCH_BYTES");
    return confidence_rows(c, sc, row_begin, n_rows, conf_out, tap_conf_out, tap_maxprob_out, tap_argmax_out, false);
}

int ssd_window_confidence(ssd_ctx* c, float* conf_out, float* tap_conf_out, int32_t* n_positions_out)
{
    if (!c || !conf_out) return c ? fail(c, SSD_EINVAL, "window_confidence: bad argument") : SSD_EINVAL;
    if (c->cfg.conf_window == 0) return fail(c, SSD_ESTATE, "window_confidence: the context was created with conf_window = 0");
    if (c->state != ST_IDLE || c->ring_count == 0) return fail(c, SSD_ESTATE, "window_confidence needs an idle prefilled sequence");
    const Dims& D = c->D;
    const Layout& Y = c->lay;
    const int R = 2 * D.L;
    const int nv = c->ring_count < c->cfg.conf_window ? (int)c->ring_count : c->cfg.conf_window;   // valid slots 0..nv-1
    const long rows = (long)nv * R;
    ConfScratch sc;
    sc.hi = c->h16(Y.hi); sc.lo = c->h16(Y.lo); sc.tapn = c->f(Y.tapn); sc.logits = c->f(Y.logits); sc.res = nullptr;
    sc.one_gemm = true;
    // rows per pass of the LM head: what the staging buffers were sized for (at least the 2L rows of one position)
    int B = rows_big_supported(D) ? SSD_PREFILL_ROWS : 64;
    if (B > Y.logit_rows) B = Y.logit_rows;
    if (B > Y.conf_rows && B > Y.rows) B = Y.conf_rows > Y.rows ? Y.conf_rows : Y.rows;
    sc.batch = B;
    float* conf_all = c->f(Y.ring_conf);                  // [nv * R], then R means
    for (long r0 = 0; r0 < rows; r0 += B) {
        const int nb = rows - r0 < B ? (int)(rows - r0) : B;
        int rc = conf_batch(c, sc, c->f(Y.ring) + (size_t)r0 * D.d, nb, conf_all + r0, nullptr, nullptr);
        if (rc) return rc;
    }
    float* means = conf_all + (size_t)c->cfg.conf_window * R;
    HIPCHK(window_mean(conf_all, nv, R, means, c->stream), "window mean");
    float hb[2 * SSD_MAX_LAYERS];
    int rc = readback(c, means, sizeof(float) * R, hb);
    if (rc) return rc;
    for (int l = 0; l < D.L; l++) {
        conf_out[l] = c->cfg.conf_taps == 2 ? 0.5f * (hb[2 * l] + hb[2 * l + 1]) : hb[2 * l + 1];
        if (tap_conf_out) { tap_conf_out[2 * l] = hb[2 * l]; tap_conf_out[2 * l + 1] = hb[2 * l + 1]; }
    }
    if (n_positions_out) *n_positions_out = nv;
    c->logit_rows = 0;  // the logits buffer was reused
    c->st.confidence_rows += rows;
    return SSD_OK;
}

int ssd_set_graphs(ssd_ctx* c, int enable)
{
    if (!c) return SSD_EINVAL;
    c->use_graphs = enable != 0;
    return SSD_OK;
}

int ssd_profile_select(ssd_ctx* c, int kernel_id)
{
    if (!c || kernel_id < -1 || kernel_id >= SSD_K_COUNT) return c ? fail(c, SSD_EINVAL, "profile_select: bad kernel id") : SSD_EINVAL;
    c->prof_kid = kernel_id;
    c->prof_used = 0;
    return SSD_OK;
}

int ssd_profile_read(ssd_ctx* c, int64_t* launches_out, double* total_ms_out)
{
    if (!c || !launches_out || !total_ms_out) return SSD_EINVAL;
    *launches_out = 0; *total_ms_out = 0.0;
    if (c->prof_used == 0) return SSD_OK;
    HIPCHK(hipStreamSynchronize(c->stream), "profile sync");
    double tot = 0.0;
    for (size_t i = 0; i < c->prof_used; i++) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, c->prof_ev[i].first, c->prof_ev[i].second), "event elapsed");
        tot += ms;
    }
    *launches_out = (int64_t)c->prof_used;
    *total_ms_out = tot;
    return SSD_OK;
}

int ssd_kv_poison_stale(ssd_ctx* c)
{
    if (!c) return SSD_EINVAL;
    if (c->state != ST_IDLE) return fail(c, SSD_ESTATE, "kv_poison_stale needs an idle prefilled sequence");
    HIPCHK(kv_poison(c->D, c->ws + c->lay.kv, c->pos_dev(), c->stream), "kv_poison");
    HIPCHK(hipStreamSynchronize(c->stream), "sync");
    return SSD_OK;
}

int ssd_hbm_read_probe(const void* dev, size_t bytes, int iters, void* hip_stream, float* ms_out)
{
    if (!dev || bytes < 16 || iters < 1 || !ms_out || reinterpret_cast<uintptr_t>(dev) % 16) return SSD_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    float* sink = nullptr;
    hipEvent_t e0, e1;
    if (hipMalloc((void**)&sink, 256) != hipSuccess) return SSD_EHIP;
    int rc = SSD_OK;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = SSD_EHIP;
    if (!rc && read_probe(dev, bytes, sink, s) != hipSuccess) rc = SSD_EHIP;  // warm-up
    if (!rc) {
        (void)hipEventRecord(e0, s);
        for (int i = 0; i < iters && !rc; i++)
            if (read_probe(dev, bytes, sink, s) != hipSuccess) rc = SSD_EHIP;
        (void)hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess) rc = SSD_EHIP;
        float ms = 0.f;
        if (!rc && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SSD_EHIP;
        *ms_out = ms / (float)iters;
    }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    return rc;
}

}  // extern "C"
