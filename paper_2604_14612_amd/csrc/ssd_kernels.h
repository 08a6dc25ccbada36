// Internal launch interface between the host state machine (ssd_api.cpp) and the gfx950
// kernels (ssd_kernels.hip).  Plain pointers and sizes only; every launcher enqueues on the
// given stream and returns the HIP status of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssdk {

enum WeightType { WT_F32 = 0, WT_BF16 = 1, WT_F16 = 2 };

// Launch options of one context: tuning hooks (0 = the library's own choice) and the one-shot request to time the
// next GEMV launch.  Owned by whoever owns the Dims that point to it; nothing here is process-global.
struct LaunchOpts {
    int gemv_block_cap = 0;     // > 0 overrides the block cap of the GEMV launches
    int gemv_resid_cfg = 0;     // residual projections: 100 R + 10 D + KS forces rows per group / steps in flight / K split
    int rows_depth = 0;         // > 0 forces the number of weight stripes a 16-row block keeps in flight
    int wide_depth = 0;         // the same for the 64-row blocks
    int gemv_cfg = 0;           // single-row GEMVs other than the residual projections: 100 R + 10 D + KS of a work split (kernel_bench sweeps)
    int wide_ksplit = 0;        // 64-row blocks: 1 = never cut K, > 1 forces the number of K slices
    int attn_splits = 0;        // > 0 forces the attention split count (scratch must have been sized for it)
    int attn_kernel = 0;        // 0 heuristic, 1 LDS-staged kernel always, 3 the same in its plain (non-MFMA) form
    // When set, the next GEMV launch records its own begin / end timestamps into the two events (kernel time as a
    // profiler reports it, without the dispatch latency a pair of stream events around the launch would include)
    // and clears the request.
    hipEvent_t time_start = nullptr, time_stop = nullptr;
};

// Shape constants shared by all launches of one context.
struct Dims {
    int L, d, H, Hkv, hd, dq, dkv, f, V, max_seq;
    float eps;
    int wt;  // WeightType of the matrices; the hi/lo activation pairs of the multi-row path use the same element type
    int kt;  // WeightType code of the KV cache elements (independent of wt)
    LaunchOpts* opt = nullptr;  // may be null: library defaults, no timing
};

// x[r][:] = embed[tok_dev[r]][:] widened to fp32 (token ids in device memory, clamped to the vocabulary).
struct TokArg { int32_t t[64]; };
hipError_t embed_rows(const Dims& D, const void* embed, const int32_t* tok_dev, int M, float* x, hipStream_t s);
// dst[i] = toks.t[i] for i < n, except dst[0] = first_dev[0] when first_dev != nullptr
hipError_t set_tokens(TokArg toks, int n, const int32_t* first_dev, int32_t* dst, hipStream_t s);

// Links of a chained launch (experimental overlap of consecutive kernels on two streams): the kernel waits, after its
// first weight loads are in flight, until *wait_flag >= wait_count * *gen, and every one of its blocks adds 1 to
// *done_flag when its outputs are visible device-wide.  Null members switch the respective half off.
struct Chain {
    unsigned* wait_flag; unsigned wait_count;
    unsigned* done_flag;
    const unsigned* gen;
    unsigned* err;
};

// ---- single-row (draft / vanilla decode) path: weight-streaming GEMV kernels ----------------
// h = rmsnorm(x, gain); q,k,v = Wq h, Wk h, Wv h; rotary on q,k at position *pos_dev + pos_off;
// q -> qbuf (fp32), k,v -> cache rows of this layer.
hipError_t gemv_qkv(const Dims& D, const void* wq, const void* wk, const void* wv, const float* gain,
                    const float* x, const float* rope, const int* pos_dev, int pos_off, float* qbuf,
                    void* kcache_l, void* vcache_l, hipStream_t s, const Chain* ch = nullptr, int* blocks_out = nullptr);
// x[n] += W[n][:] . in[:]   (N x K), optional tap copy of the updated x
hipError_t gemv_resid(const Dims& D, const void* w, int N, int K, const float* in, float* x, float* tap,
                      hipStream_t s, const Chain* ch = nullptr, int* blocks_out = nullptr);
// x += Wo . att (d x dq), att being the fold of the n_splits attention partials of a single row that
// attention() left in part when asked to defer the fold
hipError_t gemv_resid_attn(const Dims& D, const void* w, const float* part, int n_splits, float* x, float* tap,
                           hipStream_t s);
// act[n] = silu(Wg[n] . h) * (Wu[n] . h), h = rmsnorm(x, gain)
hipError_t gemv_swiglu(const Dims& D, const void* wg, const void* wu, const float* gain, const float* x,
                       float* act, hipStream_t s, const Chain* ch = nullptr, int* blocks_out = nullptr);
// logits[n] = Wlm[n] . rmsnorm(x, gain)
hipError_t gemv_lmhead(const Dims& D, const void* wlm, const float* gain, const float* x, float* logits,
                       hipStream_t s);

// The same with the vocabulary reduction of a greedy step folded in: every block also leaves (max, sum of exp,
// arg-max) of its clamped logits in vstat (3 floats per block, GEMV_MAX_BLOCKS blocks at most) and a one-block
// kernel combines them into the greedy token (lowest index among equal maxima) and its soft-max probability.
constexpr int GEMV_MAX_BLOCKS = 1024;
hipError_t gemv_lmhead_argmax(const Dims& D, const void* wlm, const float* gain, const float* x, float* logits, float clamp,
                              float* vstat, int32_t* tok_out, float* maxprob_out, hipStream_t s);

// ---- multi-row (verify / prefill / confidence) path ------------------------------------------
// out[r][:] = rmsnorm(in[r][:], gain) for r < M   (rows of length K)
hipError_t rmsnorm_rows(const float* in, const float* gain, int M, int K, float eps, float* out, hipStream_t s);
// Y[r][n] (op)= sum_k W[n][k] X[r][k], r < M <= 16.  bf16 weights use MFMA tiles, fp32 weights plain FMAs.
//   mode 0: store to y (ld = N_total), up to three stacked matrices (QKV) written side by side
//   mode 1: y += (residual add), optional tap copy (tap row stride tap_ld)
//   mode 2: y = silu(W0 x) * (W1 x)  (two matrices of n0 rows each)
struct RowsGemm {
    const void* w[3];
    int n[3];
    int K;
    const float* x;  // [M][K]
    float* y;        // [M][ldy]
    int ldy;
    float* tap;      // mode 1 only, may be null
    int tap_ld;
    int M;
    int mode;
};
hipError_t gemm_rows(const Dims& D, const RowsGemm& g, hipStream_t s);
// Multi-row MFMA GEMM for bf16 / fp16 weights with K a multiple of 64.  Activations come pre-split into
// hi/lo arrays of the same 16-bit type [M][ldb] (rows_prep, rows_gain_split, attention with out_hi/out_lo, the SwiGLU mode
// or a RESID projection with gain_out).
//   mode 0 store fp32, 1 residual add into y (+ tap), 2 SwiGLU of two matrices written as hi/lo to
//   oh/ol, 3 QKV: rotary on q and k at positions *pos_dev + pos_off + r, q -> y [M][dq] fp32,
//   k and v -> cache rows.
// RMSNorm without a kernel: a mode-1 call with gain_out set also writes split(y * gain_out) to oh/ol
// [M][ldo] and the sums of y^2 over each 16-column tile to ssq_out [M][n/16]; a mode-0/2/3 call with
// ssq set treats bh/bl as such un-normalised rows and scales its results by
// rsqrt(sum(ssq[r][0..n_ssq)) / K + eps).
struct RowsFused {
    const void* w[3];
    int n[3];
    int K;
    const uint16_t* bh; const uint16_t* bl; int ldb;
    float* y; int ldy;
    uint16_t* oh; uint16_t* ol; int ldo;
    float* tap; int tap_ld;
    int M;
    int mode;
    const float* rope; const int* pos_dev; int pos_off;
    void* kc; void* vc;
    const float* ssq; int n_ssq;
    const float* gain_out; float* ssq_out;
    float* kpart; size_t kpart_floats;  // rows_wide / rows_big: scratch for a split along K (may be null: no split)
    int tap_only;                       // > 0: only row tap_only - 1 writes its tap, into tap row 0
};
bool rows_fused_supported(const Dims& D);
hipError_t rows_fused(const Dims& D, const RowsFused& f, hipStream_t s);
// y[r][n] = sum_k W[n][k] (bh + bl)[r][k] for up to 64 pre-split rows at once (the per-layer confidence rows
// against the LM head): W is streamed once for all of them.  bf16, N a multiple of 64, K a multiple of 128.
// The same GEMMs for any number of rows in one launch, on 128 x 128 tiles (prompts, the context window): weights
// cross the chip once for all rows.  16-bit weights; d, dq, dkv, V multiples of 128, f of 64, K of 64.
bool rows_big_supported(const Dims& D);
hipError_t rows_big(const Dims& D, const RowsFused& f, hipStream_t s);
bool rows_many_supported(const Dims& D, int N, int K);
hipError_t rows_many(const Dims& D, const void* w, int N, int K, const uint16_t* bh, const uint16_t* bl, int ldb, int M,
                     float* y, int ldy, hipStream_t s);
// The modes of rows_fused for up to 64 rows per pass (prompt blocks): 64-row weight tiles, n[] multiples of 64,
// K a multiple of 128; the sums of squares it reads / writes are per 64-column tile.
bool rows_wide_supported(const Dims& D);
hipError_t rows_wide(const Dims& D, const RowsFused& f, hipStream_t s);
// hi/lo bf16 split of M rows (row stride ldx) of length K into [M][K] arrays, RMS-normalised with
// gain first when gain != nullptr
hipError_t rows_prep(const Dims& D, const float* in, int ldx, const float* gain, int M, int K, float eps, uint16_t* hi,
                     uint16_t* lo, hipStream_t s);
// hi/lo = split(in * gain) (no norm scale) and ssq[r][t] = sum of in[r][group t .. group (t+1))^2, group = 16
// (rows_fused) or 64 (rows_wide): the form in which a RESID projection with gain_out hands rows to its consumer
hipError_t rows_gain_split(const Dims& D, const float* in, int ldx, const float* gain, int M, int K, uint16_t* hi, uint16_t* lo,
                           float* ssq, int group, hipStream_t s);
// rotary on q,k rows + cache write for the multi-row path. qkv: [M][dq + 2 dkv]; q is rotated in place.
hipError_t rope_kv_rows(const Dims& D, float* qkv, const float* rope, const int* pos_dev, int pos_off, int M,
                        void* kcache_l, void* vcache_l, hipStream_t s);

// ---- attention over the KV cache ---------------------------------------------------------------
// Row r (r < M) at position p_r = *pos_dev + pos_off + r attends cache positions 0..p_r.
// q: [M][ldq] fp32 (head h at offset h*hd); out: [M][dq] fp32, or, when out_hi != nullptr, the bf16
// hi/lo pair [M][dq] instead.  part: scratch for the split partials.
hipError_t attention(const Dims& D, const float* q, int ldq, const void* kcache_l, const void* vcache_l,
                     const int* pos_dev, int pos_off, int pos_host_hint, int M, float* part, float* out,
                     uint16_t* out_hi, uint16_t* out_lo, hipStream_t s, int* deferred_splits = nullptr);
// deferred_splits (single row only): when the positions are split over several blocks the fold is left to
// the consumer; *deferred_splits = the number of partials per head to pass to gemv_resid_attn, or 0 when
// out already holds the result.
size_t attention_scratch_floats(const Dims& D, int max_rows);
// launch shape attention() uses when the last of M rows sees ctx positions: the number of position ranges,
// negated for the register-resident kernel (two calls with equal values enqueue identical launches)
int attention_splits(const Dims& D, int ctx, int M);

// ---- vocabulary reduction ------------------------------------------------------------------------
// Per row of logits [M][V]: arg-max (lowest index on ties), softmax max-probability and, when
// conf != nullptr, the entropy confidence of Eq. 1-4 (clamp applied first).  tok_out[r*tok_stride]
// receives the arg-max when tok_out != nullptr.
hipError_t vocab_reduce(const float* logits, int M, int V, float clamp, float eps, int32_t* tok_out,
                        int tok_stride, int32_t* argmax_out, float* maxprob_out, float* conf_out,
                        hipStream_t s);

// means[t] = mean over positions p < n_pos of v[p * n_taps + t] (context-window average of per-row confidences)
hipError_t window_mean(const float* v, int n_pos, int n_taps, float* means, hipStream_t s);

// ---- static scratch -----------------------------------------------------------------------------------
// A fixed-size device array inside the library image, for the one entry point that must not allocate.  Every
// device holds its own copy at its own address: static_scratch_for_device resolves it once per device (that device
// must be current) and returns the cached device pointer afterwards.  Contents persist from call to call.
size_t static_scratch_bytes();
hipError_t static_scratch_for_device(int device, void** ptr_out);

// ---- small state kernels ---------------------------------------------------------------------------
// tok0 = token, *pos_dev = pos
hipError_t set_state(int32_t* tok0, int32_t token, int* pos_dev, int pos, hipStream_t s);
// *pos_dev += delta;  tok0 = src[0] when src != nullptr
hipError_t advance_state(int* pos_dev, int delta, int32_t* tok0, const int32_t* src, hipStream_t s);
// NaN-fill cache positions >= *pos_dev of all layers
hipError_t kv_poison(const Dims& D, void* kv_all, const int* pos_dev, hipStream_t s);
// copy n floats
hipError_t copy_f32(const float* src, float* dst, size_t n, hipStream_t s);
// read-only streaming probe; *sink_dev receives a checksum so the loads cannot be dropped
hipError_t read_probe(const void* dev, size_t bytes, float* sink_dev, hipStream_t s);

}  // namespace ssdk
