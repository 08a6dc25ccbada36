// kernel_bench: runs the library's hot kernels in isolation at Llama-2-7B shapes (distinct weights for
// every launch, so nothing is served from the caches) and prints the time per launch.  Used for tuning
// and, under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`, for the HBM traffic of each kernel; the
// read probe and the fp32 copy move a known number of bytes and calibrate those counters.
// Environment switches select other runs: KB_SWEEP (launch time against size), KB_PAIR (a kernel reading what the
// kernel before it wrote), KB_LAYER (the five launches of a decode layer in sequence), KB_LONG (three seconds of
// back-to-back gate/up launches: clock drift).
#include "ssd_kernels.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define CK(x)                                                                         \
    do {                                                                              \
        hipError_t e__ = (x);                                                         \
        if (e__ != hipSuccess) {                                                      \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e__), __LINE__); \
            std::exit(1);                                                             \
        }                                                                             \
    } while (0)

using namespace ssdk;

template <typename F>
static void timeit(const char* name, double bytes, int n, F&& launch)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    float best = 1e30f;
    for (int rep = 0; rep < 3; rep++) {
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(a, 0));
        for (int i = 0; i < n; i++) launch(i);
        CK(hipEventRecord(b, 0));
        CK(hipEventSynchronize(b));
        float ms;
        CK(hipEventElapsedTime(&ms, a, b));
        if (ms < best) best = ms;
    }
    const double us = best * 1e3 / n;
    std::printf("%-28s %9.2f us per launch  %8.1f MB  %7.0f GB/s\n", name, us, bytes / 1e6, bytes / us / 1e3);
    std::fflush(stdout);
    CK(hipEventDestroy(a)); CK(hipEventDestroy(b));
}

int main(int argc, char** argv)
{
    const int M = argc > 1 ? std::atoi(argv[1]) : 5;  // rows of the multi-row kernels (k + 1)
    if (M < 1 || M > 16) { std::printf("rows must be 1..16\n"); return 1; }
    Dims D;
    D.L = 32; D.d = 4096; D.H = 32; D.Hkv = 32; D.hd = 128; D.dq = 4096; D.dkv = 4096; D.f = 11008; D.V = 32000;
    D.max_seq = 1024; D.eps = 1e-5f; D.wt = WT_BF16;
    // cache element type: the library's default (fp32) unless KB_KV=bf16
    const bool kv16 = std::getenv("KB_KV") && !std::strcmp(std::getenv("KB_KV"), "bf16");
    D.kt = kv16 ? WT_BF16 : WT_F32;
    const size_t kvb = kv16 ? 2 : 4;
    LaunchOpts opts;   // tuning hooks of this run
    D.opt = &opts;
    const size_t wbig = (size_t)3 << 30;  // 6 GB of bf16 weights to walk through
    uint16_t* W;
    CK(hipMalloc(&W, wbig * 2));
    {
        std::vector<uint16_t> h(1 << 24);
        unsigned st = 12345;
        for (auto& v : h) { st = st * 1664525u + 1013904223u; v = (uint16_t)(0x3c00 | ((st >> 16) & 0x83ff)); }
        for (size_t o = 0; o < wbig; o += h.size()) CK(hipMemcpy(W + o, h.data(), h.size() * 2, hipMemcpyHostToDevice));
    }
    float *x, *gain, *act, *q, *rope, *logits, *part, *sink, *big_a, *big_b;
    int* pos;
    char *kc, *vc;   // KV cache copies, kvb bytes per element
    uint16_t *hi, *lo, *hi64, *lo64;
    const size_t act_floats = (size_t)16 * 32000;
    CK(hipMalloc(&x, act_floats * 4)); CK(hipMalloc(&gain, 1 << 20)); CK(hipMalloc(&act, act_floats * 4));
    CK(hipMalloc(&q, act_floats * 4)); CK(hipMalloc(&logits, act_floats * 4)); CK(hipMalloc(&part, 128 << 20));
    CK(hipMalloc(&rope, (size_t)1024 * 64 * 2 * 4)); CK(hipMalloc(&pos, 64)); CK(hipMalloc(&sink, 256));
    const size_t kv_layer = (size_t)32 * 1024 * 128;  // elements of K (or V) of one layer; one copy per timed launch so the cache is cold
    CK(hipMalloc(&kc, 12 * kv_layer * kvb)); CK(hipMalloc(&vc, 12 * kv_layer * kvb));
    CK(hipMalloc(&hi, act_floats * 2)); CK(hipMalloc(&lo, act_floats * 2));
    CK(hipMalloc(&hi64, (size_t)64 * 11008 * 2)); CK(hipMalloc(&lo64, (size_t)64 * 11008 * 2));
    CK(hipMemset(hi64, 0, (size_t)64 * 11008 * 2)); CK(hipMemset(lo64, 0, (size_t)64 * 11008 * 2));
    CK(hipMalloc(&big_a, (size_t)256 << 20)); CK(hipMalloc(&big_b, (size_t)256 << 20));
    CK(hipMemset(x, 0, act_floats * 4)); CK(hipMemset(gain, 0, 1 << 20)); CK(hipMemset(act, 0, act_floats * 4));
    CK(hipMemset(q, 0, act_floats * 4)); CK(hipMemset(rope, 0, (size_t)1024 * 64 * 2 * 4));
    CK(hipMemset(kc, 0, 12 * kv_layer * kvb)); CK(hipMemset(vc, 0, 12 * kv_layer * kvb));
    CK(hipMemset(hi, 0, act_floats * 2)); CK(hipMemset(lo, 0, act_floats * 2));
    const int ctx = 640;
    CK(hipMemcpy(pos, &ctx, 4, hipMemcpyHostToDevice));
    const size_t gu = (size_t)11008 * 4096, qk = (size_t)4096 * 4096, lm = (size_t)32000 * 4096;
    const int n = 12;

    // calibration kernels: known traffic
    timeit("read_probe 256 MiB", 268435456.0, 4, [&](int i) { CK(read_probe(W + (size_t)i * (134217728), (size_t)256 << 20, sink, 0)); });
    timeit("copy_f32 256 MiB", 2 * 268435456.0, 4, [&](int) { CK(copy_f32(big_a, big_b, (size_t)64 << 20, 0)); });

    if (std::getenv("KB_LONG")) {   // sustained streaming: does the per-launch time drift once the chip has been busy for a while?
        for (int rep = 0; rep < 40; rep++) {
            hipEvent_t a, b;
            CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
            CK(hipEventRecord(a, 0));
            const int launches = 2400;
            for (int i = 0; i < launches; i++) {
                const uint16_t* w = W + (size_t)(i % 12) * 2 * gu;
                CK(gemv_swiglu(D, w, w + gu, gain, x, act, 0));
            }
            CK(hipEventRecord(b, 0)); CK(hipEventSynchronize(b));
            float ms; CK(hipEventElapsedTime(&ms, a, b));
            std::printf("gemv_gateup sustained, %d launches: %.2f us per launch\n", launches, ms * 1e3 / launches);
            std::fflush(stdout);
        }
        return 0;
    }
    if (std::getenv("KB_PAIR")) {   // a kernel that reads what the kernel before it has just written (as in the layer pipeline)
        timeit("gemv_o alone", qk * 2.0, n, [&](int i) { CK(gemv_resid(D, W + (size_t)i * qk, 4096, 4096, q, x, nullptr, 0)); });
        timeit("gemv_gateup alone", 2 * gu * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 2 * gu;
            CK(gemv_swiglu(D, w, w + gu, gain, x, act, 0)); });
        timeit("gemv_o then gemv_gateup (x handed over)", qk * 2.0 + 2 * gu * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 3 * gu;
            CK(gemv_resid(D, w + 2 * gu, 4096, 4096, q, x, nullptr, 0));
            CK(gemv_swiglu(D, w, w + gu, gain, x, act, 0)); });
        timeit("gemv_gateup then gemv_down (act handed over)", 3 * gu * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 3 * gu;
            CK(gemv_swiglu(D, w, w + gu, gain, x, act, 0));
            CK(gemv_resid(D, w + 2 * gu, 4096, 11008, act, x, nullptr, 0)); });
        return 0;
    }
    if (std::getenv("KB_LAYER")) {   // the five launches of a decode layer in sequence, 12 different layers' worth of weights
        const size_t layer_elems = 4 * qk + 3 * gu;
        timeit("decode layer: qkv, attention, o (fold), gate/up, down", layer_elems * 2.0 + 2.0 * 641 * 4096 * kvb, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * layer_elems;
            CK(gemv_qkv(D, w, w + qk, w + 2 * qk, gain, x, rope, pos, 0, q, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, 0));
            int fold = 0;
            CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, 1, part, act, nullptr, nullptr, 0,
                         &fold));
            if (fold > 0) CK(gemv_resid_attn(D, w + 3 * qk, part, fold, x, nullptr, 0));
            else CK(gemv_resid(D, w + 3 * qk, 4096, 4096, act, x, nullptr, 0));
            CK(gemv_swiglu(D, w + 4 * qk, w + 4 * qk + gu, gain, x, act, 0));
            CK(gemv_resid(D, w + 4 * qk + 2 * gu, 4096, 11008, act, x, nullptr, 0)); });
        return 0;
    }
    if (std::getenv("KB_CHAIN")) {
        // Chained launches: the four GEMVs of a layer (QKV, output projection, gate/up, down; attention left out) on
        // alternating streams, each waiting for its producer's blocks through a device counter instead of a kernel
        // boundary, against the same launches in order on one stream.
        hipStream_t sx, sy;
        CK(hipStreamCreate(&sx)); CK(hipStreamCreate(&sy));
        const size_t layer_elems = 4 * qk + 3 * gu;
        const int nl = 12, nk = 4 * nl;
        unsigned *flags, *gen, *err;
        CK(hipMalloc(&flags, (nk + 1) * sizeof(unsigned))); CK(hipMalloc(&gen, 64)); CK(hipMalloc(&err, 64));
        const unsigned one = 1;
        CK(hipMemcpy(gen, &one, 4, hipMemcpyHostToDevice)); CK(hipMemset(err, 0, 64));
        hipEvent_t e0, e1, ej;
        CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1)); CK(hipEventCreate(&ej));
        std::vector<int> blocks(nk + 1, 0);
        // meaningful data, so that the two orders can be compared: small random residual, unit gains
        std::vector<float> x0(4096), ones(4096, 1.0f), xa(4096), xb(4096);
        { unsigned st = 777; for (auto& v : x0) { st = st * 1664525u + 1013904223u; v = ((st >> 8) & 0xffff) / 65536.0f - 0.5f; } }
        CK(hipMemcpy(gain, ones.data(), 4096 * 4, hipMemcpyHostToDevice));
        auto run = [&](bool chained) {
            hipStream_t st[2] = {sx, chained ? sy : sx};
            CK(hipMemcpyAsync(x, x0.data(), 4096 * 4, hipMemcpyHostToDevice, sx));
            CK(hipMemsetAsync(flags, 0, (nk + 1) * sizeof(unsigned), sx));
            if (chained) { CK(hipEventRecord(ej, sx)); CK(hipStreamWaitEvent(sy, ej, 0)); }
            CK(hipEventRecord(e0, sx));
            int ki = 0;
            for (int l = 0; l < nl; l++) {
                const uint16_t* w = W + (size_t)l * layer_elems;
                for (int j = 0; j < 4; j++, ki++) {
                    Chain ch = {};
                    if (chained) {
                        if (ki > 0) { ch.wait_flag = flags + ki - 1; ch.wait_count = (unsigned)blocks[ki - 1]; }
                        ch.done_flag = flags + ki; ch.gen = gen; ch.err = err;
                    }
                    hipStream_t s = st[ki & 1];
                    const Chain* c = chained ? &ch : nullptr;
                    if (j == 0) CK(gemv_qkv(D, w, w + qk, w + 2 * qk, gain, x, rope, pos, 0, q, kc, vc, s, c, &blocks[ki]));
                    else if (j == 1) CK(gemv_resid(D, w + 3 * qk, 4096, 4096, q, x, nullptr, s, c, &blocks[ki]));
                    else if (j == 2) CK(gemv_swiglu(D, w + 4 * qk, w + 4 * qk + gu, gain, x, act, s, c, &blocks[ki]));
                    else CK(gemv_resid(D, w + 4 * qk + 2 * gu, 4096, 11008, act, x, nullptr, s, c, &blocks[ki]));
                }
            }
            if (chained) { CK(hipEventRecord(ej, sy)); CK(hipStreamWaitEvent(sx, ej, 0)); }
            CK(hipEventRecord(e1, sx));
            CK(hipEventSynchronize(e1));
            float ms; CK(hipEventElapsedTime(&ms, e0, e1));
            return ms * 1e3 / nl;
        };
        for (int rep = 0; rep < 6; rep++) {
            // Two chained kernels must fit the chip together (a waiting consumer must never hold the slots its
            // producer's remaining blocks need): each gets at most half of the 768 resident block slots.
            const int cap = rep < 2 ? 384 : rep < 4 ? 256 : 320;
            opts.gemv_block_cap = 0;
            const double a = run(false);
            CK(hipMemcpy(xa.data(), x, 4096 * 4, hipMemcpyDeviceToHost));
            opts.gemv_block_cap = cap;
            const double b = run(true);
            opts.gemv_block_cap = 0;
            CK(hipMemcpy(xb.data(), x, 4096 * 4, hipMemcpyDeviceToHost));
            unsigned e = 0; CK(hipMemcpy(&e, err, 4, hipMemcpyDeviceToHost));
            int diff = 0; double mag = 0;
            for (int i = 0; i < 4096; i++) { diff += std::memcmp(&xa[i], &xb[i], 4) != 0; mag += std::fabs(xa[i]); }
            std::printf("GEMVs of a layer (qkv, o, gate/up, down): one stream %.2f us, chained on two streams (block cap %d) %.2f us per layer, "
                        "wait timeouts %u, residual elements that differ %d of 4096 (mean |x| %.3g)\n", a, cap, b, e, diff, mag / 4096);
            std::fflush(stdout);
        }
        return 0;
    }
    if (std::getenv("KB_WARM")) {
        // Does a GEMV run faster on weights that a plain read kernel has just pulled through the 256 MB memory-side
        // cache?  (If it did, a prefetcher running ahead of the launch sequence could hide launch gaps.)  Every timed
        // launch is preceded by a read of 1 GB of other data; "warm" re-reads the matrix with plain loads first.
        hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
        for (int rows : {4096, 8192, 11008, 16384, 22016}) {
            const size_t bytes = (size_t)rows * 4096 * 2;
            for (int mode = 0; mode < 3; mode++) {   // 0 cold GEMV, 1 GEMV after a plain-load read of the matrix, 2 plain-load read after the same
                float tot = 0.f;
                const int reps = 10;
                for (int r = 0; r < reps + 1; r++) {
                    const uint16_t* w = W + (size_t)(r % 10) * ((size_t)96 << 20);
                    CK(read_probe(W + ((size_t)2 << 30), (size_t)1 << 30, sink, 0));
                    if (mode) CK(copy_f32((const float*)w, big_a, bytes / 4, 0));   // plain loads (and 1x the bytes written elsewhere)
                    CK(hipEventRecord(a, 0));
                    if (mode == 2) CK(copy_f32((const float*)w, big_b, bytes / 4, 0));
                    else CK(gemv_resid(D, w, rows, 4096, q, logits, nullptr, 0));
                    CK(hipEventRecord(b, 0)); CK(hipEventSynchronize(b));
                    float ms; CK(hipEventElapsedTime(&ms, a, b));
                    if (r) tot += ms;   // the first repetition warms the code path
                }
                const char* nm[3] = {"GEMV, cold", "GEMV after a plain read of the same matrix", "plain copy after a plain read (for scale)"};
                std::printf("%6d x 4096 (%6.1f MB)  %-44s %8.2f us\n", rows, bytes / 1e6, nm[mode], tot * 1e3 / reps);
                std::fflush(stdout);
            }
        }
        return 0;
    }
    if (std::getenv("KB_RESID")) {   // residual projections (output 4096 x 4096, down 4096 x 11008): work split sweep
        const int ctx1 = 640;
        for (int cfg : {0, 241, 242, 244, 248, 222, 224, 228, 422, 424, 428, 442, 444}) for (int cap : {0, 512, 1024}) {
            opts.gemv_resid_cfg = cfg; opts.gemv_block_cap = cap;
            char nm[96];
            std::snprintf(nm, sizeof nm, "gemv_o cfg %d cap %d", cfg, cap);
            timeit(nm, qk * 2.0, n, [&](int i) { CK(gemv_resid(D, W + (size_t)i * qk, 4096, 4096, q, x, nullptr, 0)); });
            std::snprintf(nm, sizeof nm, "gemv_down cfg %d cap %d", cfg, cap);
            timeit(nm, gu * 2.0, n, [&](int i) { CK(gemv_resid(D, W + (size_t)i * gu, 4096, 11008, act, x, nullptr, 0)); });
            std::snprintf(nm, sizeof nm, "attention + gemv_o (fold) cfg %d cap %d", cfg, cap);
            timeit(nm, 2.0 * (ctx1 + 1) * 4096 * kvb + qk * 2.0, n, [&](int i) {
                int fold = 0;
                CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx1, 1, part, act, nullptr, nullptr,
                             0, &fold));
                if (fold > 0) CK(gemv_resid_attn(D, W + (size_t)i * qk, part, fold, x, nullptr, 0));
                else CK(gemv_resid(D, W + (size_t)i * qk, 4096, 4096, act, x, nullptr, 0)); });
        }
        return 0;
    }
    if (std::getenv("KB_GEMV")) {   // QKV, gate/up and LM-head GEMVs: work split (rows per wave, steps in flight, K split) x block cap
        for (int cfg : {0, 281, 441, 421, 221, 242}) for (int cap : {0, 512, 1024}) {
            opts.gemv_cfg = cfg; opts.gemv_block_cap = cap;
            char nm[96];
            std::snprintf(nm, sizeof nm, "gemv_qkv cfg %d cap %d", cfg, cap);
            timeit(nm, 3 * qk * 2.0, n, [&](int i) {
                const uint16_t* w = W + (size_t)i * 3 * qk;
                CK(gemv_qkv(D, w, w + qk, w + 2 * qk, gain, x, rope, pos, 0, q, kc, vc, 0)); });
            std::snprintf(nm, sizeof nm, "gemv_gateup cfg %d cap %d", cfg, cap);
            timeit(nm, 2 * gu * 2.0, n, [&](int i) {
                const uint16_t* w = W + (size_t)i * 2 * gu;
                CK(gemv_swiglu(D, w, w + gu, gain, x, act, 0)); });
            std::snprintf(nm, sizeof nm, "gemv_lmhead cfg %d cap %d", cfg, cap);
            timeit(nm, lm * 2.0, n, [&](int i) { CK(gemv_lmhead(D, W + (size_t)i * lm, gain, x, logits, 0)); });
        }
        return 0;
    }
    if (std::getenv("KB_SWEEP")) {   // launch time against size: fixed cost and streaming rate of probe and GEMV
        for (int mb : {16, 32, 64, 128, 256}) {
            char nm[64];
            std::snprintf(nm, sizeof nm, "read_probe %d MiB", mb);
            timeit(nm, (double)mb * 1048576.0, 8, [&](int i) { CK(read_probe(W + (size_t)i * (134217728), (size_t)mb << 20, sink, 0)); });
        }
        for (int rows : {2048, 4096, 8192, 16384, 32768}) {
            char nm[64];
            std::snprintf(nm, sizeof nm, "gemv_resid %d x 4096", rows);
            timeit(nm, rows * 8192.0, 8, [&](int i) { CK(gemv_resid(D, W + (size_t)i * lm, rows, 4096, q, logits, nullptr, 0)); });
        }
        for (int rows : {2048, 4096, 8192, 16384, 32000}) {
            char nm[64];
            Dims D2 = D; D2.V = rows;
            std::snprintf(nm, sizeof nm, "gemv_lmhead %d x 4096", rows);
            timeit(nm, rows * 8192.0, 8, [&](int i) { CK(gemv_lmhead(D2, W + (size_t)i * lm, gain, x, logits, 0)); });
        }
        return 0;
    }
    if (std::getenv("KB_BIG")) {
        // whole-prompt GEMMs: one launch of the large-tile kernel (256 or 128 weight rows x 128 rows) over R rows against R / 64 launches of the 64-row
        // kernel (flops: one bf16 product per weight and row; the kernels do two, hi and lo)
        const int pad = std::getenv("KB_PAD") ? std::atoi(std::getenv("KB_PAD")) : 0;   // extra elements per activation row
        std::printf("activation row pitch = K + %d elements\n", pad);
        const int only_r = std::getenv("KB_BIG_R") ? std::atoi(std::getenv("KB_BIG_R")) : 0;   // one row count only
        opts.wide_depth = std::getenv("KB_TN") ? std::atoi(std::getenv("KB_TN")) : 0;   // weight rows per tile: 128, 256, 0 = library's choice
        std::printf("weight rows per tile: %d (0 = the library's choice)\n", opts.wide_depth);
        opts.wide_ksplit = std::getenv("KB_KS") ? std::atoi(std::getenv("KB_KS")) : 0;   // K slices: 1 = never, > 1 forced, 0 = library's choice
        std::printf("K slices: %d (0 = the library's choice)\n", opts.wide_ksplit);
        for (int R : {128, 256, 512, 1024}) {
            if (only_r && R != only_r) continue;
            uint16_t *bh, *bl, *oh, *ol;
            const size_t rb = (size_t)R * (11008 + pad) * 2;
            CK(hipMalloc(&bh, rb)); CK(hipMalloc(&bl, rb)); CK(hipMalloc(&oh, rb)); CK(hipMalloc(&ol, rb));
            CK(hipMemset(bh, 0, rb)); CK(hipMemset(bl, 0, rb));
            float* ssq_out;
            CK(hipMalloc(&ssq_out, (size_t)R * 64 * 4));
            auto run = [&](bool big, int mode, const uint16_t* w0, const uint16_t* w1, const uint16_t* w2, int n0, int n1, int n2, int K,
                           float* y, int ldy, int rows, int row0) {
                RowsFused f = {};
                f.w[0] = w0; f.w[1] = w1; f.w[2] = w2; f.n[0] = n0; f.n[1] = n1; f.n[2] = n2; f.K = K;
                f.bh = bh + (size_t)row0 * (K + pad); f.bl = bl + (size_t)row0 * (K + pad); f.ldb = K + pad; f.y = y ? y + (size_t)row0 * ldy : nullptr; f.ldy = ldy;
                f.oh = oh + (size_t)row0 * 11008; f.ol = ol + (size_t)row0 * 11008; f.ldo = 11008; f.M = rows; f.mode = mode;
                // (the position on the device is 640 and the cache holds 1024: the larger row counts write positions 0 .. rows - 1)
                f.rope = rope; f.pos_dev = pos; f.pos_off = 640 + rows > 1024 ? -640 : 0; f.kc = kc; f.vc = vc;
                f.kpart = part; f.kpart_floats = (size_t)32 << 20;
                if (mode != 1) { f.ssq = gain; f.n_ssq = K / 64; }
                CK(big ? rows_big(D, f, 0) : rows_wide(D, f, 0));
            };
            struct Shape { const char* name; int mode; size_t welems; int n0, n1, n2, K, ldy; };
            const Shape shapes[] = {{"qkv", 3, 3 * qk, 4096, 4096, 4096, 4096, 4096}, {"o (resid)", 1, qk, 4096, 0, 0, 4096, 4096},
                                    {"gateup (swiglu)", 2, 2 * gu, 11008, 11008, 0, 4096, 0}, {"down (resid)", 1, gu, 4096, 0, 0, 11008, 4096},
                                    {"lmhead (store)", 0, lm, 32000, 0, 0, 4096, 32000}};
            for (const Shape& sh : shapes) {
                const double flops = 2.0 * (double)sh.welems * R;
                for (int big = 1; big >= 0; big--) {
                    char nm[96];
                    std::snprintf(nm, sizeof nm, "%s %4d rows, %s", sh.name, R, big ? "large tiles, 1 launch" : "64-row kernel per 64 rows");
                    hipEvent_t a, b;
                    CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
                    float best = 1e30f;
                    for (int rep = 0; rep < 3; rep++) {
                        CK(hipDeviceSynchronize());
                        CK(hipEventRecord(a, 0));
                        for (int i = 0; i < 4; i++) {
                            const uint16_t* w = W + (size_t)i * sh.welems;
                            const uint16_t* w1 = sh.mode == 3 ? w + qk : sh.mode == 2 ? w + gu : nullptr;
                            const uint16_t* w2 = sh.mode == 3 ? w + 2 * qk : nullptr;
                            float* y = sh.mode == 2 ? nullptr : big_a;
                            if (big) run(true, sh.mode, w, w1, w2, sh.n0, sh.n1, sh.n2, sh.K, y, sh.ldy, R, 0);
                            else for (int r0 = 0; r0 < R; r0 += 64) run(false, sh.mode, w, w1, w2, sh.n0, sh.n1, sh.n2, sh.K, y, sh.ldy, 64, r0);
                        }
                        CK(hipEventRecord(b, 0));
                        CK(hipEventSynchronize(b));
                        float ms;
                        CK(hipEventElapsedTime(&ms, a, b));
                        if (ms < best) best = ms;
                    }
                    const double us = best * 1e3 / 4;
                    std::printf("%-52s %9.1f us  %7.1f TFLOP/s\n", nm, us, flops / us / 1e6);
                    std::fflush(stdout);
                    CK(hipEventDestroy(a)); CK(hipEventDestroy(b));
                }
            }
            CK(hipFree(bh)); CK(hipFree(bl)); CK(hipFree(oh)); CK(hipFree(ol)); CK(hipFree(ssq_out));
        }
        return 0;
    }
    if (std::getenv("KB_COUNTERS")) {
        // Every kernel of a decode layer and of a verify layer once per line, in the library's own configuration and
        // nothing else: under `rocprofv3 --pmc` a kernel name (plus grid size) then maps to exactly one of these lines.
        timeit("gemv_qkv", 3 * qk * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 3 * qk;
            CK(gemv_qkv(D, w, w + qk, w + 2 * qk, gain, x, rope, pos, 0, q, kc, vc, 0)); });
        timeit("attention 1 row ctx 641 + gemv_o folding its partials", 2.0 * 641 * 4096 * kvb + qk * 2.0, n, [&](int i) {
            int fold = 0;
            CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, 1, part, act, nullptr, nullptr,
                         0, &fold));
            if (fold > 0) CK(gemv_resid_attn(D, W + (size_t)i * qk, part, fold, x, nullptr, 0));
            else CK(gemv_resid(D, W + (size_t)i * qk, 4096, 4096, act, x, nullptr, 0)); });
        timeit("gemv_gateup (swiglu)", 2 * gu * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 2 * gu;
            CK(gemv_swiglu(D, w, w + gu, gain, x, act, 0)); });
        timeit("gemv_down (resid)", gu * 2.0, n, [&](int i) { CK(gemv_resid(D, W + (size_t)i * gu, 4096, 11008, act, x, nullptr, 0)); });
        timeit("gemv_lmhead", lm * 2.0, n, [&](int i) { CK(gemv_lmhead(D, W + (size_t)i * lm, gain, x, logits, 0)); });
        auto rows = [&](int mode, const uint16_t* w0, const uint16_t* w1, const uint16_t* w2, int n0, int n1, int n2, int K,
                        float* y, int ldy) {
            RowsFused f = {};
            f.w[0] = w0; f.w[1] = w1; f.w[2] = w2; f.n[0] = n0; f.n[1] = n1; f.n[2] = n2; f.K = K;
            f.bh = hi; f.bl = lo; f.ldb = K; f.y = y; f.ldy = ldy; f.oh = hi; f.ol = lo; f.ldo = 11008; f.M = M; f.mode = mode;
            f.rope = rope; f.pos_dev = pos; f.pos_off = 0; f.kc = kc; f.vc = vc;
            if (mode != 1) { f.ssq = gain; f.n_ssq = K / 16; }
            CK(rows_fused(D, f, 0));
        };
        timeit("rows_qkv", 3 * qk * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 3 * qk;
            rows(3, w, w + qk, w + 2 * qk, 4096, 4096, 4096, 4096, q, 4096); });
        timeit("attention M rows ctx 640+M (MFMA kernel + fold)", 2.0 * (640 + M) * 4096 * kvb, n, [&](int i) {
            CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, M, part, nullptr, hi,
                         lo, 0)); });
        timeit("rows_o (resid)", qk * 2.0, n, [&](int i) { rows(1, W + (size_t)i * qk, nullptr, nullptr, 4096, 0, 0, 4096, x, 4096); });
        timeit("rows_gateup (swiglu)", 2 * gu * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 2 * gu;
            rows(2, w, w + gu, nullptr, 11008, 11008, 0, 4096, nullptr, 0); });
        timeit("rows_down (resid)", gu * 2.0, n, [&](int i) { rows(1, W + (size_t)i * gu, nullptr, nullptr, 4096, 0, 0, 11008, x, 4096); });
        timeit("rows_lmhead", lm * 2.0, n, [&](int i) { rows(0, W + (size_t)i * lm, nullptr, nullptr, 32000, 0, 0, 4096, logits, 32000); });
        auto wide64 = [&](int mode, const uint16_t* w0, const uint16_t* w1, const uint16_t* w2, int n0, int n1, int n2, int K,
                          float* y, int ldy) {
            RowsFused f = {};
            f.w[0] = w0; f.w[1] = w1; f.w[2] = w2; f.n[0] = n0; f.n[1] = n1; f.n[2] = n2; f.K = K;
            f.bh = hi64; f.bl = lo64; f.ldb = K; f.y = y; f.ldy = ldy; f.oh = hi64; f.ol = lo64; f.ldo = 11008; f.M = 64; f.mode = mode;
            f.rope = rope; f.pos_dev = pos; f.pos_off = 0; f.kc = kc; f.vc = vc;
            f.kpart = part; f.kpart_floats = (size_t)16 << 20;
            CK(rows_wide(D, f, 0));
        };
        timeit("wide_qkv (64 rows)", 3 * qk * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 3 * qk;
            wide64(3, w, w + qk, w + 2 * qk, 4096, 4096, 4096, 4096, big_a, 4096); });
        timeit("wide_o (64 rows)", qk * 2.0, n, [&](int i) { wide64(1, W + (size_t)i * qk, nullptr, nullptr, 4096, 0, 0, 4096, big_b, 4096); });
        timeit("wide_gateup (64 rows)", 2 * gu * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 2 * gu;
            wide64(2, w, w + gu, nullptr, 11008, 11008, 0, 4096, nullptr, 0); });
        timeit("wide_down (64 rows)", gu * 2.0, n, [&](int i) { wide64(1, W + (size_t)i * gu, nullptr, nullptr, 4096, 0, 0, 11008, big_b, 4096); });
        timeit("rows_many lmhead 64 rows", lm * 2.0, n, [&](int i) {
            CK(rows_many(D, W + (size_t)i * lm, 32000, 4096, hi64, lo64, 4096, 64, big_a, 32000, 0)); });
        timeit("attention 64 rows ctx 640+64 (MFMA kernel + fold)", 2.0 * (640 + 64) * 4096 * kvb, n, [&](int i) {
            CK(attention(D, big_a, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, 64, part, nullptr,
                         hi64, lo64, 0)); });
        {   // a whole prompt of 512 rows at positions 0..511 through the large-tile kernel
            const int R = 512;
            uint16_t *bh, *bl, *oh, *ol;
            int* pos0;
            const size_t rb = (size_t)R * 11008 * 2;
            CK(hipMalloc(&bh, rb)); CK(hipMalloc(&bl, rb)); CK(hipMalloc(&oh, rb)); CK(hipMalloc(&ol, rb)); CK(hipMalloc(&pos0, 64));
            CK(hipMemset(bh, 0, rb)); CK(hipMemset(bl, 0, rb)); CK(hipMemset(pos0, 0, 64));
            auto big = [&](int mode, const uint16_t* w0, const uint16_t* w1, const uint16_t* w2, int n0, int n1, int n2, int K,
                           float* y, int ldy) {
                RowsFused f = {};
                f.w[0] = w0; f.w[1] = w1; f.w[2] = w2; f.n[0] = n0; f.n[1] = n1; f.n[2] = n2; f.K = K;
                f.bh = bh; f.bl = bl; f.ldb = K; f.y = y; f.ldy = ldy; f.oh = oh; f.ol = ol; f.ldo = 11008; f.M = R; f.mode = mode;
                f.rope = rope; f.pos_dev = pos0; f.pos_off = 0; f.kc = kc; f.vc = vc;
                f.kpart = part; f.kpart_floats = (size_t)16 << 20;
                if (mode != 1) { f.ssq = gain; f.n_ssq = K / 64; }
                CK(rows_big(D, f, 0));
            };
            timeit("big_qkv (512 rows)", 3 * qk * 2.0, n, [&](int i) {
                const uint16_t* w = W + (size_t)i * 3 * qk;
                big(3, w, w + qk, w + 2 * qk, 4096, 4096, 4096, 4096, big_a, 4096); });
            timeit("big_o (512 rows)", qk * 2.0, n, [&](int i) { big(1, W + (size_t)i * qk, nullptr, nullptr, 4096, 0, 0, 4096, big_b, 4096); });
            timeit("big_gateup (512 rows)", 2 * gu * 2.0, n, [&](int i) {
                const uint16_t* w = W + (size_t)i * 2 * gu;
                big(2, w, w + gu, nullptr, 11008, 11008, 0, 4096, nullptr, 0); });
            timeit("big_down (512 rows)", gu * 2.0, n, [&](int i) { big(1, W + (size_t)i * gu, nullptr, nullptr, 4096, 0, 0, 11008, big_b, 4096); });
            timeit("big_lmhead (512 rows)", lm * 2.0, n, [&](int i) { big(0, W + (size_t)i * lm, nullptr, nullptr, 32000, 0, 0, 4096, big_a, 32000); });
        }
        return 0;
    }
    // single-row (draft / vanilla decode) kernels
    for (int cap : {0, 1024, 512}) {
    opts.gemv_block_cap = cap;
    std::printf("-- gemv block cap %d\n", cap);
    timeit("gemv_qkv", 3 * qk * 2.0, n, [&](int i) {
        const uint16_t* w = W + (size_t)i * 3 * qk;
        CK(gemv_qkv(D, w, w + qk, w + 2 * qk, gain, x, rope, pos, 0, q, kc, vc, 0)); });
    timeit("gemv_o (resid)", qk * 2.0, n, [&](int i) { CK(gemv_resid(D, W + (size_t)i * qk, 4096, 4096, q, x, nullptr, 0)); });
    timeit("gemv_gateup (swiglu)", 2 * gu * 2.0, n, [&](int i) {
        const uint16_t* w = W + (size_t)i * 2 * gu;
        CK(gemv_swiglu(D, w, w + gu, gain, x, act, 0)); });
    timeit("gemv_down (resid)", gu * 2.0, n, [&](int i) { CK(gemv_resid(D, W + (size_t)i * gu, 4096, 11008, act, x, nullptr, 0)); });
    timeit("gemv_lmhead", lm * 2.0, n, [&](int i) { CK(gemv_lmhead(D, W + (size_t)i * lm, gain, x, logits, 0)); });
    }
    opts.gemv_block_cap = 0;
    for (int kind : {1, 0}) {   // 1 = LDS-staged kernel forced, 0 = launch plan (register-resident kernel for few queries)
        opts.attn_kernel = kind;
        for (int sp : {0, 1, 2, 4, 8}) {
            if (kind == 1 && sp != 0 && sp < 8) continue;   // the LDS-staged kernel needs ctx / 96 ranges at least
            opts.attn_splits = sp;
            char nm[96];
            std::snprintf(nm, sizeof nm, "attention 1 row ctx 641, %s, splits %s%d", kind ? "lds-staged" : "planned",
                          sp ? "" : "auto=", sp ? sp : std::abs(attention_splits(D, ctx + 1, 1)));
            timeit(nm, 2.0 * 641 * 4096 * kvb, n, [&](int i) {
                CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, 1, part, act, nullptr,
                             nullptr, 0)); });
        }
    }
    opts.attn_splits = 0;
    opts.attn_kernel = 0;
    timeit("attention + gemv_o, fold kernel", 2.0 * 641 * 4096 * kvb + qk * 2.0, n, [&](int i) {
        CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, 1, part, act, nullptr, nullptr, 0));
        CK(gemv_resid(D, W + (size_t)i * qk, 4096, 4096, act, x, nullptr, 0)); });
    for (int cap : {0, 512}) for (int sp : {0, 4, 8}) {
        opts.attn_splits = sp;
        opts.gemv_block_cap = cap;
        char nm[96];
        std::snprintf(nm, sizeof nm, "attention + gemv_o, fold in gemv, splits %d cap %d", sp, cap);
        timeit(nm, 2.0 * 641 * 4096 * kvb + qk * 2.0, n, [&](int i) {
            int fold = 0;
            CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, 1, part, act, nullptr, nullptr,
                         0, &fold));
            if (fold > 0) CK(gemv_resid_attn(D, W + (size_t)i * qk, part, fold, x, nullptr, 0));
            else CK(gemv_resid(D, W + (size_t)i * qk, 4096, 4096, act, x, nullptr, 0)); });
    }
    opts.attn_splits = 0;
    opts.gemv_block_cap = 0;
    timeit("vocab_reduce 1 row", 32000 * 4.0, n, [&](int) {
        CK(vocab_reduce(logits, 1, 32000, 1e4f, 1e-10f, pos + 8, 1, nullptr, sink, nullptr, 0)); });

    // multi-row (verify) kernels, M rows
    bool with_ssq = false;
    auto fused = [&](int mode, const uint16_t* w0, const uint16_t* w1, const uint16_t* w2, int n0, int n1, int n2, int K,
                     float* y, int ldy) {
        RowsFused f = {};
        f.w[0] = w0; f.w[1] = w1; f.w[2] = w2; f.n[0] = n0; f.n[1] = n1; f.n[2] = n2; f.K = K;
        f.bh = hi; f.bl = lo; f.ldb = K; f.y = y; f.ldy = ldy; f.oh = hi; f.ol = lo; f.ldo = 11008; f.M = M; f.mode = mode;
        f.rope = rope; f.pos_dev = pos; f.pos_off = 0; f.kc = kc; f.vc = vc;
        if (with_ssq && mode != 1) { f.ssq = gain; f.n_ssq = K / 16; }   // gain is a zeroed 1 MB buffer: values do not matter here
        CK(rows_fused(D, f, 0));
    };
    if (std::getenv("KB_ROWS")) {   // 16-row kernels: weight stripes in flight per block
        with_ssq = true;
        for (int dpt : {0, 1, 2, 3, 4}) {
            opts.rows_depth = dpt;
            std::printf("-- 16-row kernels, %d rows, stripes in flight %d (0 = library's choice)\n", M, dpt);
            timeit("rows_qkv", 3 * qk * 2.0, n, [&](int i) {
                const uint16_t* w = W + (size_t)i * 3 * qk;
                fused(3, w, w + qk, w + 2 * qk, 4096, 4096, 4096, 4096, q, 4096); });
            timeit("rows_o (resid)", qk * 2.0, n, [&](int i) { fused(1, W + (size_t)i * qk, nullptr, nullptr, 4096, 0, 0, 4096, x, 4096); });
            timeit("rows_gateup (swiglu)", 2 * gu * 2.0, n, [&](int i) {
                const uint16_t* w = W + (size_t)i * 2 * gu;
                fused(2, w, w + gu, nullptr, 11008, 11008, 0, 4096, nullptr, 0); });
            timeit("rows_down (resid)", gu * 2.0, n, [&](int i) { fused(1, W + (size_t)i * gu, nullptr, nullptr, 4096, 0, 0, 11008, x, 4096); });
            timeit("rows_lmhead", lm * 2.0, n, [&](int i) { fused(0, W + (size_t)i * lm, nullptr, nullptr, 32000, 0, 0, 4096, logits, 32000); });
        }
        opts.rows_depth = 0;
        return 0;
    }
    for (int v : {0, 1}) {
    with_ssq = v != 0;
    std::printf("-- 16-row kernels%s\n", v ? ", consumers summing 256 sum-of-squares partials per row (RMSNorm folded in)" : "");
    timeit("rows_prep (norm+split)", M * 4096 * 8.0, n, [&](int) { CK(rows_prep(D, x, 4096, gain, M, 4096, 1e-5f, hi, lo, 0)); });
    timeit("rows_qkv", 3 * qk * 2.0, n, [&](int i) {
        const uint16_t* w = W + (size_t)i * 3 * qk;
        fused(3, w, w + qk, w + 2 * qk, 4096, 4096, 4096, 4096, q, 4096); });
    timeit("rows_o (resid)", qk * 2.0, n, [&](int i) { fused(1, W + (size_t)i * qk, nullptr, nullptr, 4096, 0, 0, 4096, x, 4096); });
    timeit("rows_gateup (swiglu)", 2 * gu * 2.0, n, [&](int i) {
        const uint16_t* w = W + (size_t)i * 2 * gu;
        fused(2, w, w + gu, nullptr, 11008, 11008, 0, 4096, nullptr, 0); });
    timeit("rows_down (resid)", gu * 2.0, n, [&](int i) { fused(1, W + (size_t)i * gu, nullptr, nullptr, 4096, 0, 0, 11008, x, 4096); });
    timeit("rows_lmhead", lm * 2.0, n, [&](int i) { fused(0, W + (size_t)i * lm, nullptr, nullptr, 32000, 0, 0, 4096, logits, 32000); });
    }
    for (int rows : {16, 64}) {
        char nm[96];
        std::snprintf(nm, sizeof nm, "rows_many lmhead %d rows", rows);
        timeit(nm, lm * 2.0, n, [&](int i) {
            CK(rows_many(D, W + (size_t)i * lm, 32000, 4096, hi, lo, 4096, rows, big_a, 32000, 0)); });
    }
    {
        const int M0 = M;
        (void)M0;
        auto wide = [&](int mode, const uint16_t* w0, const uint16_t* w1, const uint16_t* w2, int n0, int n1, int n2, int K,
                        float* y, int ldy) {
            RowsFused f = {};
            f.w[0] = w0; f.w[1] = w1; f.w[2] = w2; f.n[0] = n0; f.n[1] = n1; f.n[2] = n2; f.K = K;
            f.bh = hi64; f.bl = lo64; f.ldb = K; f.y = y; f.ldy = ldy; f.oh = hi64; f.ol = lo64; f.ldo = 11008; f.M = 64; f.mode = mode;
            f.rope = rope; f.pos_dev = pos; f.pos_off = 0; f.kc = kc; f.vc = vc;
            f.kpart = part; f.kpart_floats = (size_t)16 << 20;
            CK(rows_wide(D, f, 0));
        };
        for (int ks : {0, 1, 2, 4, 8}) {
        opts.wide_ksplit = ks;
        std::printf("-- 64-row pass (prompt blocks), K slices: %d (0 = library's choice, 1 = none)\n", ks);
        timeit("wide_qkv", 3 * qk * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 3 * qk;
            wide(3, w, w + qk, w + 2 * qk, 4096, 4096, 4096, 4096, big_a, 4096); });
        timeit("wide_o (resid)", qk * 2.0, n, [&](int i) { wide(1, W + (size_t)i * qk, nullptr, nullptr, 4096, 0, 0, 4096, big_b, 4096); });
        timeit("wide_gateup (swiglu)", 2 * gu * 2.0, n, [&](int i) {
            const uint16_t* w = W + (size_t)i * 2 * gu;
            wide(2, w, w + gu, nullptr, 11008, 11008, 0, 4096, nullptr, 0); });
        timeit("wide_down (resid)", gu * 2.0, n, [&](int i) { wide(1, W + (size_t)i * gu, nullptr, nullptr, 4096, 0, 0, 11008, big_b, 4096); });
        }
        opts.wide_ksplit = 0;
    }
    for (int kind : {1, 0}) {
        opts.attn_kernel = kind;
        for (int sp : {0, 2, 4, 8, 16}) {
            if (kind == 1 && sp != 0) continue;
            opts.attn_splits = sp;
            char nm[96];
            std::snprintf(nm, sizeof nm, "attention M rows ctx 640+M, %s, splits %s%d", kind ? "lds-staged" : "planned",
                          sp ? "" : "auto=", sp ? sp : std::abs(attention_splits(D, ctx + M, M)));
            timeit(nm, 2.0 * (640 + M) * 4096 * kvb, n, [&](int i) {
                CK(attention(D, q, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, M, part, nullptr, hi,
                             lo, 0)); });
        }
    }
    opts.attn_splits = 0;
    opts.attn_kernel = 0;
    for (int kind : {3, 1}) for (int rows : {9, 16, 64}) for (int sp : {0, 16}) {
        if (sp && (kind == 3 || rows != 64)) continue;
        opts.attn_kernel = kind;
        opts.attn_splits = sp;
        char nm[96];
        std::snprintf(nm, sizeof nm, "attention %d rows ctx 640+rows, LDS-staged %s, splits %d", rows, kind == 3 ? "plain" : "MFMA", sp);
        timeit(nm, 2.0 * (640 + rows) * 4096 * kvb, n, [&](int i) {
            CK(attention(D, big_a, 4096, kc + (size_t)i * kv_layer * kvb, vc + (size_t)i * kv_layer * kvb, pos, 0, ctx, rows, part, nullptr,
                         hi64, lo64, 0)); });
    }
    opts.attn_kernel = 0;
    opts.attn_splits = 0;
    return 0;
}
