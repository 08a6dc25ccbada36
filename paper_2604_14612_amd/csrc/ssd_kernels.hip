// gfx950 (CDNA4, wave64) kernels of the self-speculative decoding hot path.
//
// Single-row path (draft model of Section 3 and vanilla decoding): weight-streaming GEMV kernels for
// bf16 / fp16 / fp32 weights -- every lane issues 128-bit loads along K, fp32 FMAs against the
// activation vector held in LDS, wave-shuffle reduction; RMSNorm is fused into the prologue, rotary
// embedding + KV-cache write / residual add / SwiGLU into the epilogues.  Attention over the cache
// runs out of registers on ranges of ~128 positions; the output projection folds the range partials.
// Multi-row path (verification of k+1 rows, prompt rows, per-layer confidence rows): the same
// weight stream, staged through LDS, feeds 16x16x32 MFMA tiles; activations enter as an exact hi+lo
// split of their fp32 values in the weights' 16-bit type, and RMSNorm is folded into the epilogue
// of the producing and the consuming projection.  Models whose shapes do not fit the MFMA tiling
// (and fp32 models) take a plain FMA path with separate norm / rotary kernels.
#include "ssd_kernels.h"

#include <hip/hip_ext.h>

#include <math.h>

#include <algorithm>
#include <atomic>
#include <mutex>

namespace ssdk {

// ---------------------------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);   // round to nearest even; gfx950 converts in hardware
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int VEC = 4;  // elements per 128-bit load
    __device__ static __forceinline__ void load(const float* p, float (&o)[4])
    {
        float4 v = *reinterpret_cast<const float4*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    __device__ static __forceinline__ float get(const float* p, size_t i) { return p[i]; }
    __device__ static __forceinline__ void put(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct Elem<uint16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ void load(const uint16_t* p, float (&o)[8])
    {
        uint4 v = *reinterpret_cast<const uint4*>(p);
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
        o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
        o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    __device__ static __forceinline__ float get(const uint16_t* p, size_t i) { return bf16_bits_to_f32(p[i]); }
    __device__ static __forceinline__ void put(uint16_t* p, size_t i, float v) { p[i] = f32_to_bf16_bits(v); }
};

typedef _Float16 f16_t;   // IEEE binary16 storage (weights and cache of fp16 models)
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
template <> struct Elem<f16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ void load(const f16_t* p, float (&o)[8])
    {
        const f16x8_t v = *reinterpret_cast<const f16x8_t*>(p);
#pragma unroll
        for (int i = 0; i < 8; i++) o[i] = (float)v[i];
    }
    __device__ static __forceinline__ float get(const f16_t* p, size_t i) { return (float)p[i]; }
    __device__ static __forceinline__ void put(f16_t* p, size_t i, float v) { p[i] = (f16_t)v; }  // round to nearest even
};
template <typename T> struct IsF16 { static constexpr bool value = false; };
template <> struct IsF16<f16_t> { static constexpr bool value = true; };

// one 16-bit storage element (bf16 or fp16 bit pattern) from an fp32 value
__device__ __forceinline__ uint16_t f32_to_h16_bits(float v, bool f16)
{
    if (f16) return __builtin_bit_cast(uint16_t, (f16_t)v);
    return f32_to_bf16_bits(v);
}
__device__ __forceinline__ float h16_bits_to_f32(uint16_t h, bool f16)
{
    if (f16) return (float)__builtin_bit_cast(f16_t, h);
    return bf16_bits_to_f32(h);
}

// one KV-cache element of type kt (WeightType code) from an fp32 value, round to nearest even
__device__ __forceinline__ void kv_put(void* base, size_t i, float v, int kt)
{
    if (kt == WT_F32) reinterpret_cast<float*>(base)[i] = v;
    else if (kt == WT_F16) reinterpret_cast<f16_t*>(base)[i] = (f16_t)v;
    else reinterpret_cast<uint16_t*>(base)[i] = f32_to_bf16_bits(v);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Block-wide sum for blocks of NW waves; red must hold NW floats. All threads get the result.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red)
{
    v = wave_sum(v);
    int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; i++) t += red[i];
    return t;
}

// Block barrier for data exchanged through LDS only: waits for this wave's LDS operations and then for the other
// waves.  __syncthreads() also carries a fence that waits for every global load in flight (loads and stores share
// one counter on this architecture), which would drain a register prefetch at every staging step; a loaded register
// is still protected by the wait the compiler places before its first use.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------------------------------------
// embedding gather
// ---------------------------------------------------------------------------------------------
template <typename WT>
__global__ void embed_kernel(const WT* __restrict__ E, const int32_t* __restrict__ tok_dev, int d, int V,
                             float* __restrict__ x)
{
    int r = blockIdx.y;
    int t = tok_dev[r];
    t = min(max(t, 0), V - 1);
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < d; i += gridDim.x * blockDim.x)
        x[(size_t)r * d + i] = Elem<WT>::get(E, (size_t)t * d + i);
}

hipError_t embed_rows(const Dims& D, const void* embed, const int32_t* tok_dev, int M, float* x, hipStream_t s)
{
    dim3 grid(ceil_div(D.d, 256), M);
    if (D.wt == WT_BF16)
        hipLaunchKernelGGL(embed_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t*)embed, tok_dev, D.d, D.V, x);
    else if (D.wt == WT_F16)
        hipLaunchKernelGGL(embed_kernel<f16_t>, grid, dim3(256), 0, s, (const f16_t*)embed, tok_dev, D.d, D.V, x);
    else
        hipLaunchKernelGGL(embed_kernel<float>, grid, dim3(256), 0, s, (const float*)embed, tok_dev, D.d, D.V, x);
    return hipGetLastError();
}

__global__ void set_tokens_kernel(TokArg toks, int n, const int32_t* first_dev, int32_t* dst)
{
    int i = threadIdx.x;
    if (i < n) dst[i] = (i == 0 && first_dev) ? first_dev[0] : toks.t[i];
}
hipError_t set_tokens(TokArg toks, int n, const int32_t* first_dev, int32_t* dst, hipStream_t s)
{
    hipLaunchKernelGGL(set_tokens_kernel, dim3(1), dim3(64), 0, s, toks, n, first_dev, dst);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// single-row weight-streaming GEMV
// ---------------------------------------------------------------------------------------------
// A block has 8 waves.  KS consecutive waves form a group that owns R "logical" weight rows;
// the K dimension is cut into chunks of one 128-bit load per lane (512 bf16 / 256 fp32) and the
// waves of a group take chunks kp, kp+KS, ...  Every wave keeps D chunk-steps of R non-temporal
// loads in flight (weights are read exactly once, they should not displace activations in the
// caches).  The input vector sits in LDS already multiplied by the norm gain; the RMS scale is a
// per-vector scalar and is applied to the finished dot products.
// Logical row order: QKV interleaves the two rows of a rotary pair (i, i + hd/2), gate/up
// interleaves gate row n and up row n, so that one lane holds both operands of the epilogue.
constexpr int GV_WAVES = 8;
constexpr int GV_THREADS = GV_WAVES * 64;
constexpr int GV_FOLD_MAX = 8;  // attention partials per head the output projection can fold itself

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_STORE = 3 };

struct GemvP {
    const void* w0; const void* w1; const void* w2;
    const float* in;    // [K]
    const float* part;  // when set (RESID only): the input is the fold of n_splits attention partials of row 0
    int n_splits;       //   laid out [K / hd heads][n_splits][hd + 4] as the attention kernels write them
    const float* gain;  // rmsnorm gain or nullptr (input used as is)
    float eps;
    int K;
    int n_rows;         // logical rows (QKV: dq + 2 dkv; SWIGLU: 2 f; else N)
    float* y;           // QKV: qbuf; RESID: residual (+=); SWIGLU: act; STORE: logits
    float* tap;
    void* kc; void* vc; int kt;   // cache rows of this layer and their element type (WeightType code)
    const float* rope;  // [max_seq][hd/2][2] (cos, sin)
    const int* pos_dev; int pos_off;
    int hd, dq, dkv, max_seq;
    float* vstat;       // STORE only, may be null: per block (max, sum of exp relative to it, arg-max) of the clamped outputs
    float clamp;
    // Chained launches (all null / 0 = an ordinary launch).  A chained kernel may start while its producer is still
    // running: it issues its first weight loads, then waits until *wait_flag has reached wait_count * *gen (every
    // block of the producer adds 1 to its done_flag once its outputs are visible device-wide), and only then reads
    // its input vector -- with device-coherent loads, as the producer's stores were device-coherent write-throughs.
    unsigned* wait_flag; unsigned wait_count;
    unsigned* done_flag;
    const unsigned* gen;     // replay generation (1, 2, ...): the counters are never reset
    unsigned* err;           // set to 1 if a wait gave up (every wait is bounded)
};

// Device-coherent accesses for data handed from one running kernel to another (each XCD has its own L2: ordinary
// loads may hit a stale line, ordinary stores stay in the writer's L2 until its kernel ends).
__device__ __forceinline__ float coh_load(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float4 coh_load4(const float* p)   // p 16-byte aligned
{
    const unsigned long long a = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long b = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p) + 1, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return make_float4(__uint_as_float((unsigned)a), __uint_as_float((unsigned)(a >> 32)), __uint_as_float((unsigned)b),
                       __uint_as_float((unsigned)(b >> 32)));
}
__device__ __forceinline__ void coh_store(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
constexpr int CHAIN_SPIN_MAX = 1 << 20;   // polls before a chained wait gives up (seconds; a healthy wait takes microseconds)

// Block-wide wait for the producer of a chained launch.  Ends for certain: the poll count is bounded.
__device__ __forceinline__ void chain_wait(const GemvP& p)
{
    if (p.wait_flag) {
        if (threadIdx.x == 0) {
            const unsigned target = p.wait_count * p.gen[0];
            int spins = 0;
            // The counter is polled with a read-modify-write (adding 0): device-scope RMW atomics are carried out at
            // the memory side, whereas a load may keep hitting a stale line in this XCD's L2.
            while (__hip_atomic_fetch_add(p.wait_flag, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                if (++spins >= CHAIN_SPIN_MAX) { __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
                __builtin_amdgcn_s_sleep(4);
            }
            // one acquire per block: drops this CU's L1 and the XCD's stale L2 lines before the inputs are read
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        __syncthreads();
    }
}
// Block-wide signal at the end of a chained launch: all of the block's write-through stores have been acknowledged.
__device__ __forceinline__ void chain_signal(const GemvP& p)
{
    if (p.done_flag) {
        __builtin_amdgcn_s_waitcnt(0);   // vmcnt(0): this wave's stores have completed
        __syncthreads();
        if (threadIdx.x == 0) __hip_atomic_fetch_add(p.done_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

template <typename WT> __device__ __forceinline__ u32x4_t gv_load(const WT* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
}

// LDS position of element i of the staged input vector.  With 8 elements per lane (16-bit weights) a chunk of 512
// elements is stored as two planes of 64 float4: plane 0 holds elements 8 l .. 8 l + 3 of lane l, plane 1 elements
// 8 l + 4 .. 8 l + 7, so that each of a wave's two 128-bit reads covers 1 KB of consecutive LDS (in natural order the
// lanes are 32 bytes apart and every read has two-way bank conflicts: measured 1.6-2 us of a 32 us launch).
template <int VEC> __device__ __forceinline__ int gv_xpos(int i)
{
    if (VEC != 8) return i;
    return (i & ~511) + ((i >> 2) & 1) * 256 + ((i & 511) >> 3) * 4 + (i & 3);
}
constexpr int GV_XB = 256;   // floats between a lane's two float4 (16-bit weights)
constexpr int GV_RES_ROUNDS = 8;   // rounds of a block whose residual values are staged in LDS (later rounds read memory)

// acc += w . x for one 128-bit weight vector; xs points at the lane's activations of this chunk in LDS
template <typename WT> __device__ __forceinline__ float gv_dot(u32x4_t w, const float* xs, float acc);
template <> __device__ __forceinline__ float gv_dot<uint16_t>(u32x4_t w, const float* xs, float acc)
{
    float4 a = *reinterpret_cast<const float4*>(xs), b = *reinterpret_cast<const float4*>(xs + GV_XB);
    acc = fmaf(__uint_as_float(w.x << 16), a.x, acc);
    acc = fmaf(__uint_as_float(w.x & 0xffff0000u), a.y, acc);
    acc = fmaf(__uint_as_float(w.y << 16), a.z, acc);
    acc = fmaf(__uint_as_float(w.y & 0xffff0000u), a.w, acc);
    acc = fmaf(__uint_as_float(w.z << 16), b.x, acc);
    acc = fmaf(__uint_as_float(w.z & 0xffff0000u), b.y, acc);
    acc = fmaf(__uint_as_float(w.w << 16), b.z, acc);
    acc = fmaf(__uint_as_float(w.w & 0xffff0000u), b.w, acc);
    return acc;
}
template <> __device__ __forceinline__ float gv_dot<f16_t>(u32x4_t w, const float* xs, float acc)
{
    const f16x8_t h = __builtin_bit_cast(f16x8_t, w);
    float4 a = *reinterpret_cast<const float4*>(xs), b = *reinterpret_cast<const float4*>(xs + GV_XB);
    acc = fmaf((float)h[0], a.x, acc); acc = fmaf((float)h[1], a.y, acc);
    acc = fmaf((float)h[2], a.z, acc); acc = fmaf((float)h[3], a.w, acc);
    acc = fmaf((float)h[4], b.x, acc); acc = fmaf((float)h[5], b.y, acc);
    acc = fmaf((float)h[6], b.z, acc); acc = fmaf((float)h[7], b.w, acc);
    return acc;
}
template <> __device__ __forceinline__ float gv_dot<float>(u32x4_t w, const float* xs, float acc)
{
    float4 a = *reinterpret_cast<const float4*>(xs);
    acc = fmaf(__uint_as_float(w.x), a.x, acc);
    acc = fmaf(__uint_as_float(w.y), a.y, acc);
    acc = fmaf(__uint_as_float(w.z), a.z, acc);
    acc = fmaf(__uint_as_float(w.w), a.w, acc);
    return acc;
}

template <typename WT, int EPI>
__device__ __forceinline__ const WT* gv_row_ptr(const GemvP& p, int j)
{
    if (EPI == EPI_QKV) {
        if (j < p.dq + p.dkv) {
            const WT* base = (const WT*)p.w0;
            int jj = j;
            if (j >= p.dq) { base = (const WT*)p.w1; jj = j - p.dq; }
            const int head = jj / p.hd, e = jj % p.hd;
            const int i = (e >> 1) + (e & 1) * (p.hd >> 1);
            return base + (size_t)(head * p.hd + i) * p.K;
        }
        return (const WT*)p.w2 + (size_t)(j - p.dq - p.dkv) * p.K;
    } else if (EPI == EPI_SWIGLU) {
        return ((j & 1) ? (const WT*)p.w1 : (const WT*)p.w0) + (size_t)(j >> 1) * p.K;
    } else {
        return (const WT*)p.w0 + (size_t)j * p.K;
    }
}

// running soft-max statistics of the rows a lane has finished: maximum, its lowest row index, sum of exp(v - max)
struct VStat { float m; float z; int arg; };
__device__ __forceinline__ void vstat_add(VStat& a, float v, int idx)
{
    if (v > a.m) { a.z = a.z * __expf(a.m - v) + 1.0f; a.m = v; a.arg = idx; }   // first row: exp(-inf) = 0
    else a.z += __expf(v - a.m);
}
// merge b into a; equal maxima keep the lower index
__device__ __forceinline__ void vstat_merge(VStat& a, const VStat& b)
{
    if (b.m > a.m || (b.m == a.m && b.arg < a.arg)) {
        a.z = (a.m > -INFINITY ? a.z * __expf(a.m - b.m) : 0.f) + b.z;
        a.m = b.m; a.arg = b.arg;
    } else if (b.m > -INFINITY) {
        a.z += b.z * __expf(b.m - a.m);
    }
}

// finished sums s[0..R) of logical rows j0.. ; sc = RMS scale (1 when no norm).  What the epilogue reads besides its
// sums comes out of LDS, staged by the kernel's prologue -- the rotary row of the position (rope_row, QKV) and the
// residual values of the group (res, null = read them from memory) -- so that no memory load sits between the steps
// of the weight pipeline (a load there has to be waited for together with every weight load in flight).
template <typename WT, int EPI, int R>
__device__ __forceinline__ void gv_epilogue(const GemvP& p, int j0, const float (&s)[R], float sc, VStat& vs, int pos,
                                            const float* rope_row, const float* res)
{
    if (EPI == EPI_QKV) {
        const int half = p.hd >> 1;
#pragma unroll
        for (int t = 0; t < R; t += 2) {
            const int j = j0 + t;
            const float a = s[t] * sc, b = s[t + 1] * sc;
            if (j < p.dq + p.dkv) {
                const bool is_q = j < p.dq;
                const int jj = is_q ? j : j - p.dq;
                const int head = jj / p.hd, i = (jj % p.hd) >> 1;
                const float* cs = rope_row + i * 2;
                const float c = cs[0], sn = cs[1];
                const float ra = a * c - b * sn, rb = b * c + a * sn;
                if (is_q) {
                    float* q = p.y + (size_t)head * p.hd + i;
                    if (p.done_flag) { coh_store(q, ra); coh_store(q + half, rb); }
                    else { q[0] = ra; q[half] = rb; }
                } else {
                    const size_t o = ((size_t)head * p.max_seq + pos) * p.hd + i;
                    kv_put(p.kc, o, ra, p.kt);
                    kv_put(p.kc, o + half, rb, p.kt);
                }
            } else {
                const int e = j - p.dq - p.dkv;
                const size_t o = ((size_t)(e / p.hd) * p.max_seq + pos) * p.hd + (e % p.hd);
                kv_put(p.vc, o, a, p.kt);
                kv_put(p.vc, o + 1, b, p.kt);
            }
        }
    } else if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int t = 0; t < R; t += 2) {
            const float g = s[t] * sc, u = s[t + 1] * sc;
            const float a = g / (1.0f + __expf(-g)) * u;
            if (p.done_flag) coh_store(p.y + ((j0 + t) >> 1), a);
            else p.y[(j0 + t) >> 1] = a;
        }
    } else if (EPI == EPI_RESID) {
#pragma unroll
        for (int t = 0; t < R; t++) {
            // chained: the residual was written by a kernel that may still have been running when this one started
            const float v = (res ? res[t] : p.wait_flag ? coh_load(p.y + j0 + t) : p.y[j0 + t]) + s[t];
            if (p.done_flag) coh_store(p.y + j0 + t, v);
            else p.y[j0 + t] = v;
            if (p.tap) p.tap[j0 + t] = v;
        }
    } else {
#pragma unroll
        for (int t = 0; t < R; t++) {
            const float v = s[t] * sc;
            p.y[j0 + t] = v;
            if (p.vstat) vstat_add(vs, fminf(fmaxf(v, -p.clamp), p.clamp), j0 + t);   // rows arrive in ascending order
        }
    }
}

template <typename WT, int EPI, int R, int D, int KS>
__global__ __launch_bounds__(GV_THREADS) void gemv_kernel(GemvP p)
{
    extern __shared__ __align__(16) float xs[];
    __shared__ float red[GV_WAVES];
    __shared__ float part[GV_WAVES][R];
    __shared__ float rope_row[EPI == EPI_QKV ? 128 : 1];                                  // (cos, sin) pairs of the position
    __shared__ float res_s[EPI == EPI_RESID ? GV_WAVES * GV_RES_ROUNDS * R : 1];          // [group slot][round][row]
    constexpr int VEC = Elem<WT>::VEC, CH = 64 * VEC, GPB = GV_WAVES / KS;
    const int lane = threadIdx.x & 63;
    // made wave-uniform for the compiler: group numbers and row pointers stay in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int grp = wave / KS, kp = wave % KS;
    const int K = p.K;
    const int n_groups = p.n_rows / R;
    const int nfull = K / CH, tail = K - nfull * CH;   // tail is a multiple of VEC
    // A row is NCH chunks of one load step, the last one partial when tail > 0 (lanes past the row's end are masked).
    // Wave kp owns chunks kp, kp + KS, ..: S steps per group, the same for every wave of the block so that block
    // barriers stay uniform.
    const int NCH = nfull + (tail > 0 ? 1 : 0);
    const int S = (NCH + KS - 1) / KS;
    const int n_gblocks = (n_groups + GPB - 1) / GPB;
    const int n_rounds = (n_gblocks - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int T = n_rounds * S;   // this wave's items (group, step), walked in order
    const int lv_full = lane * VEC;
    const int lv_tail = tail > 0 ? min(lane * VEC, tail - VEC) : 0;   // lanes past a partial chunk re-read its last vector
    const bool lane_in_tail = lane * VEC < tail;

    // Issue side of the software pipeline: D items ahead of the consume side, across groups.  Every issue is
    // UNCONDITIONAL -- a slot past the last group re-reads the last group, a step past the last chunk re-reads the last
    // chunk, and such items are never consumed.  With conditional loads the compiler cannot count what is in flight and
    // waits for everything, the loads just issued included, before every step: one memory latency per step.
    // The waves of a launch start together and their rows lie a multiple of the memory channels' interleave apart:
    // where a wave owns whole rows (KS = 1), group g walks its chunks starting at its (g mod S_kp)-th one and wraps
    // around, so that the waves are spread over the row (and the channels) from the first step on; waves that share a
    // row start at different chunks anyway (measured: the rotation gains 4 % on the 7B LM head, 10 % on the 70B one, and
    // loses 1-3 % where waves share rows; a start at (block / 8) mod S_kp, which is what helps the 16-row kernel, loses
    // up to 15 % here).
    // S_kp = chunks this wave owns.
    const int S_kp = kp < NCH ? (NCH - kp + KS - 1) / KS : 0;
    int ri = 0, ci = 0, rot_i = 0;
    const WT* wi[R];
    auto set_issue_rows = [&]() {
        int g = ((int)blockIdx.x + min(ri, max(n_rounds - 1, 0)) * (int)gridDim.x) * GPB + grp;
        g = min(g, n_groups - 1);
        rot_i = (KS == 1 && S_kp > 0) ? g % S_kp : 0;
#pragma unroll
        for (int r = 0; r < R; r++) wi[r] = gv_row_ptr<WT, EPI>(p, g * R + r);
    };
    set_issue_rows();
    u32x4_t buf[D][R];
    auto issue = [&](int s) {
        int j = ci + rot_i;
        if (j >= S_kp) j -= S_kp;
        const int c = ci < S_kp ? kp + j * KS : NCH - 1;   // (a step past the wave's last chunk re-reads the row's last chunk)
        const size_t off = (size_t)c * CH + (c == nfull ? lv_tail : lv_full);
#pragma unroll
        for (int r = 0; r < R; r++) buf[s][r] = gv_load(wi[r] + off);
        if (++ci == S) { ci = 0; ++ri; set_issue_rows(); }
    };
    // the first weight loads do not depend on the activations: start them before staging the input
#pragma unroll
    for (int s = 0; s < D; s++) issue(s);

    chain_wait(p);
    // stage the input vector (times gain); the sum of squares gives the RMS scale
    float ss = 0.f;
    if (EPI == EPI_RESID && p.part) {
        // attention output folded on the fly: out = sum_s e^(m_s - m) o_s / sum_s e^(m_s - m) l_s per head.
        // All partials of an element are fetched by independent, unconditional loads (index clamped, weight
        // zeroed past n_splits) so that the fold costs one cache round trip, not one per partial.
        const int hs = p.hd + 4, ns = p.n_splits;
        for (int i = threadIdx.x * 4; i < K; i += GV_THREADS * 4) {
            const float* base = p.part + (size_t)(i / p.hd) * ns * hs;
            const int d = i % p.hd;
            float mm[GV_FOLD_MAX], ll[GV_FOLD_MAX];
            float4 oo[GV_FOLD_MAX];
#pragma unroll
            for (int sp = 0; sp < GV_FOLD_MAX; sp++) {
                const float* ps = base + min(sp, ns - 1) * hs;
                mm[sp] = ps[p.hd];
                ll[sp] = ps[p.hd + 1];
                oo[sp] = *reinterpret_cast<const float4*>(ps + d);
            }
            float gm = -INFINITY;
#pragma unroll
            for (int sp = 0; sp < GV_FOLD_MAX; sp++) gm = fmaxf(gm, mm[sp]);   // clamped duplicates do not change the max
            float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
            float den = 0.f;
#pragma unroll
            for (int sp = 0; sp < GV_FOLD_MAX; sp++) {
                const float w = (sp < ns && ll[sp] > 0.f) ? __expf(mm[sp] - gm) : 0.f;
                num.x = fmaf(w, oo[sp].x, num.x); num.y = fmaf(w, oo[sp].y, num.y);
                num.z = fmaf(w, oo[sp].z, num.z); num.w = fmaf(w, oo[sp].w, num.w);
                den = fmaf(w, ll[sp], den);
            }
            *reinterpret_cast<float4*>(xs + gv_xpos<VEC>(i)) = make_float4(num.x / den, num.y / den, num.z / den, num.w / den);
        }
    } else
    for (int i = threadIdx.x * 4; i < K; i += GV_THREADS * 4) {
        float4 v = p.wait_flag ? coh_load4(p.in + i) : *reinterpret_cast<const float4*>(p.in + i);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        if (p.gain) {
            const float4 g = *reinterpret_cast<const float4*>(p.gain + i);
            v.x *= g.x; v.y *= g.y; v.z *= g.z; v.w *= g.w;
        }
        *reinterpret_cast<float4*>(xs + gv_xpos<VEC>(i)) = v;
    }
    int pos = 0;
    if (EPI == EPI_QKV) {
        pos = p.pos_dev[0] + p.pos_off;
        if ((int)threadIdx.x < p.hd) rope_row[threadIdx.x] = p.rope[(size_t)pos * p.hd + threadIdx.x];   // hd / 2 pairs
    }
    if (EPI == EPI_RESID) {
        for (int i = threadIdx.x; i < GPB * GV_RES_ROUNDS * R; i += GV_THREADS) {
            const int r = i % R, rnd = (i / R) % GV_RES_ROUNDS, gs = i / (R * GV_RES_ROUNDS);
            const int g = ((int)blockIdx.x + rnd * (int)gridDim.x) * GPB + gs;
            if (rnd < n_rounds && g < n_groups)
                res_s[(gs * GV_RES_ROUNDS + rnd) * R + r] = p.wait_flag ? coh_load(p.y + g * R + r) : p.y[g * R + r];
        }
    }
    float sc = 1.0f;
    if (p.gain) {
        ss = wave_sum(ss);
        if (lane == 0) red[wave] = ss;
    }
    __syncthreads();
    if (p.gain) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < GV_WAVES; i++) t += red[i];
        sc = 1.0f / sqrtf(t / (float)K + p.eps);
    }

    const float* xp = xs + (size_t)kp * CH + lane * (VEC == 8 ? 4 : VEC);   // the lane's first float4 of chunk kp
    VStat vs = {-INFINITY, 0.f, 0x7fffffff};
    int rc = 0, cc = 0;
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; r++) acc[r] = 0.f;
    auto consume = [&](int s) {
        if (rc < n_rounds) {   // uniform over the block; false only for the padding items behind the last group
            const int g = ((int)blockIdx.x + rc * (int)gridDim.x) * GPB + grp;
            const bool act = g < n_groups;
            int j = cc + ((KS == 1 && S_kp > 0) ? g % S_kp : 0);   // the issue side's chunk order
            if (j >= S_kp) j -= S_kp;
            const int c = kp + j * KS;
            if (act && cc < S_kp && (c < nfull || lane_in_tail)) {
#pragma unroll
                for (int r = 0; r < R; r++) acc[r] = gv_dot<WT>(buf[s][r], xp + (size_t)j * KS * CH, acc[r]);
            }
            if (++cc == S) {  // group finished
#pragma unroll
                for (int r = 0; r < R; r++) acc[r] = wave_sum(acc[r]);
                const float* res = (EPI == EPI_RESID && rc < GV_RES_ROUNDS) ? res_s + (grp * GV_RES_ROUNDS + rc) * R : nullptr;
                if (KS == 1) {
                    if (act && lane == 0) gv_epilogue<WT, EPI, R>(p, g * R, acc, sc, vs, pos, rope_row, res);
                } else {
                    if (lane == 0) {
#pragma unroll
                        for (int r = 0; r < R; r++) part[wave][r] = acc[r];
                    }
                    __syncthreads();
                    if (act && kp == 0 && lane == 0) {
                        float sm[R];
#pragma unroll
                        for (int r = 0; r < R; r++) {
                            float t = 0.f;
#pragma unroll
                            for (int j = 0; j < KS; j++) t += part[grp * KS + j][r];
                            sm[r] = t;
                        }
                        gv_epilogue<WT, EPI, R>(p, g * R, sm, sc, vs, pos, rope_row, res);
                    }
                    __syncthreads();
                }
#pragma unroll
                for (int r = 0; r < R; r++) acc[r] = 0.f;
                cc = 0;
                ++rc;
            }
        }
    };
    // steady state: every step consumes the oldest item and refills its slot; the last D items are consumed without
    // a refill (the item count is padded to a multiple of D: padding items are re-reads that are not consumed)
    const int Tp = (T + D - 1) / D * D;
    for (int t = 0; t + D < Tp; t += D) {
#pragma unroll
        for (int s = 0; s < D; s++) {
            consume(s);
            issue(s);
        }
    }
#pragma unroll
    for (int s = 0; s < D; s++) consume(s);
    chain_signal(p);
    if (EPI == EPI_STORE && p.vstat) {   // block partial of the soft-max statistics: lane 0 of every wave holds one
        __shared__ float vred[GV_WAVES * 3];
        if (lane == 0) { vred[wave * 3] = vs.m; vred[wave * 3 + 1] = vs.z; vred[wave * 3 + 2] = __int_as_float(vs.arg); }
        __syncthreads();
        if (threadIdx.x == 0) {
            VStat a = {vred[0], vred[1], __float_as_int(vred[2])};
#pragma unroll
            for (int w = 1; w < GV_WAVES; w++) {
                const VStat b = {vred[w * 3], vred[w * 3 + 1], __float_as_int(vred[w * 3 + 2])};
                vstat_merge(a, b);
            }
            p.vstat[blockIdx.x * 3] = a.m; p.vstat[blockIdx.x * 3 + 1] = a.z; p.vstat[blockIdx.x * 3 + 2] = __int_as_float(a.arg);
        }
    }
}

// Combines the per-block statistics of an LM-head launch: arg-max (lowest index among equal maxima) and the
// soft-max probability of that token, 1 / sum exp(z - max).
__global__ __launch_bounds__(256) void vocab_finish_kernel(const float* __restrict__ vstat, int n_blocks, int32_t* tok_out,
                                                           float* maxprob_out)
{
    __shared__ float sm[256 * 3];
    VStat a = {-INFINITY, 0.f, 0x7fffffff};
    for (int i = threadIdx.x; i < n_blocks; i += 256) {
        const VStat b = {vstat[i * 3], vstat[i * 3 + 1], __float_as_int(vstat[i * 3 + 2])};
        vstat_merge(a, b);
    }
    sm[threadIdx.x * 3] = a.m; sm[threadIdx.x * 3 + 1] = a.z; sm[threadIdx.x * 3 + 2] = __int_as_float(a.arg);
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            VStat x = {sm[threadIdx.x * 3], sm[threadIdx.x * 3 + 1], __float_as_int(sm[threadIdx.x * 3 + 2])};
            const int j = threadIdx.x + o;
            const VStat y = {sm[j * 3], sm[j * 3 + 1], __float_as_int(sm[j * 3 + 2])};
            vstat_merge(x, y);
            sm[threadIdx.x * 3] = x.m; sm[threadIdx.x * 3 + 1] = x.z; sm[threadIdx.x * 3 + 2] = __int_as_float(x.arg);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (tok_out) tok_out[0] = __float_as_int(sm[2]);
        if (maxprob_out) maxprob_out[0] = 1.0f / sm[1];
    }
}

// Largest dynamic LDS size a kernel has been enabled for.  A process-wide cache of an idempotent runtime call
// (hipFuncSetAttribute): concurrent contexts may both make the call, never skip it wrongly.
static hipError_t ensure_lds(const void* fn, size_t lds, std::atomic<size_t>& limit)
{
    if (lds <= 64 * 1024 || lds <= limit.load(std::memory_order_acquire)) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    size_t cur = limit.load(std::memory_order_relaxed);
    while (cur < lds && !limit.compare_exchange_weak(cur, lds, std::memory_order_release)) {}
    return hipSuccess;
}

// blocks_out (may be null) receives the grid size of the launch
template <typename WT, int EPI, int R, int D, int KS>
static hipError_t launch_gemv_cfg(const GemvP& p, hipStream_t s, LaunchOpts* opt, int* blocks_out)
{
    constexpr int CHF = 64 * Elem<WT>::VEC;   // the staged vector is laid out in whole chunks of one load step
    size_t lds = (size_t)ceil_div(p.K, CHF) * CHF * sizeof(float);
    static std::atomic<size_t> lds_limit{0};  // per instantiation
    {
        hipError_t e = ensure_lds((const void*)gemv_kernel<WT, EPI, R, D, KS>, lds, lds_limit);
        if (e != hipSuccess) return e;
    }
    constexpr int GPB = GV_WAVES / KS;
    int blocks = ceil_div(p.n_rows / R, GPB);
    // up to four blocks fit a CU (registers: eight waves per SIMD; LDS: the staged vector): persistent blocks that are
    // all resident at once leave no second, partial round of blocks.  Measured: three per CU are best for the
    // layer's GEMVs, four for the LM head.  The variant that folds attention partials in its prologue re-reads them
    // per block, so it runs one block per CU.
    const int per_cu = (int)std::min<size_t>(EPI == EPI_STORE ? 4 : 3, std::max<size_t>(1, ((size_t)160 << 10) / (lds + 1024)));
    int cap = p.part ? 256 : 256 * per_cu;
    if (opt && opt->gemv_block_cap > 0) cap = opt->gemv_block_cap;
    if (blocks > cap) {
        // equal work per block: with r rounds needed, use just enough blocks for r full rounds (gate/up at 7B:
        // 1376 block-rounds -> 688 blocks x 2 rather than 768 blocks of which 160 would do one round only)
        const int rounds = ceil_div(blocks, cap);
        blocks = ceil_div(blocks, rounds);
    }
    if (blocks_out) *blocks_out = blocks;
    if (opt && opt->time_start) {
        // timing request for this one launch: the events take the kernel's own begin and end timestamps
        hipExtLaunchKernelGGL((gemv_kernel<WT, EPI, R, D, KS>), dim3(blocks), dim3(GV_THREADS), lds, s, opt->time_start,
                              opt->time_stop, 0, p);
        opt->time_start = nullptr;
        opt->time_stop = nullptr;
    } else {
        hipLaunchKernelGGL((gemv_kernel<WT, EPI, R, D, KS>), dim3(blocks), dim3(GV_THREADS), lds, s, p);
    }
    return hipGetLastError();
}

// Work split: many rows -> one wave per row pair, deep pipeline; few rows -> split K over the waves
// of a group so that every wave still has a handful of chunks and the chip has thousands of waves.
template <typename WT, int EPI>
static hipError_t launch_gemv_t(const GemvP& p, hipStream_t s, LaunchOpts* opt, int* blocks_out)
{
    const int ch = ceil_div(p.K, 64 * Elem<WT>::VEC);
    if constexpr (EPI == EPI_RESID && sizeof(WT) == 2) {   // tuning hook (kernel_bench sweeps)
        switch (opt ? opt->gemv_resid_cfg : 0) {
            case 241: return launch_gemv_cfg<WT, EPI, 2, 4, 1>(p, s, opt, blocks_out);
            case 242: return launch_gemv_cfg<WT, EPI, 2, 4, 2>(p, s, opt, blocks_out);
            case 244: return launch_gemv_cfg<WT, EPI, 2, 4, 4>(p, s, opt, blocks_out);
            case 248: return launch_gemv_cfg<WT, EPI, 2, 4, 8>(p, s, opt, blocks_out);
            case 222: return launch_gemv_cfg<WT, EPI, 2, 2, 2>(p, s, opt, blocks_out);
            case 224: return launch_gemv_cfg<WT, EPI, 2, 2, 4>(p, s, opt, blocks_out);
            case 228: return launch_gemv_cfg<WT, EPI, 2, 2, 8>(p, s, opt, blocks_out);
            case 422: return launch_gemv_cfg<WT, EPI, 4, 2, 2>(p, s, opt, blocks_out);
            case 424: return launch_gemv_cfg<WT, EPI, 4, 2, 4>(p, s, opt, blocks_out);
            case 428: return launch_gemv_cfg<WT, EPI, 4, 2, 8>(p, s, opt, blocks_out);
            case 442: return launch_gemv_cfg<WT, EPI, 4, 4, 2>(p, s, opt, blocks_out);
            case 444: return launch_gemv_cfg<WT, EPI, 4, 4, 4>(p, s, opt, blocks_out);
            default: break;
        }
    }
    if constexpr (EPI != EPI_RESID && sizeof(WT) == 2) {   // tuning hook (kernel_bench sweeps)
        switch (opt ? opt->gemv_cfg : 0) {
            case 281: return launch_gemv_cfg<WT, EPI, 2, 8, 1>(p, s, opt, blocks_out);
            case 441: return launch_gemv_cfg<WT, EPI, 4, 4, 1>(p, s, opt, blocks_out);
            case 421: return launch_gemv_cfg<WT, EPI, 4, 2, 1>(p, s, opt, blocks_out);
            case 221: return launch_gemv_cfg<WT, EPI, 2, 2, 1>(p, s, opt, blocks_out);
            case 242: return launch_gemv_cfg<WT, EPI, 2, 4, 2>(p, s, opt, blocks_out);
            default: break;
        }
    }
    // measured (work-split sweeps at the 7B shape, `KB_GEMV=1` / `KB_RESID=1 kernel_bench`): row pairs with four steps
    // in flight everywhere; QKV and gate/up gain 0.5-0.8 us from two waves sharing a pair, the down projection 0.4 us
    // from four, the LM head and the projection that folds the attention partials are best with a wave per pair
    if (p.n_rows >= 8192) {
        if constexpr (sizeof(WT) == 2 && (EPI == EPI_QKV || EPI == EPI_SWIGLU)) return launch_gemv_cfg<WT, EPI, 2, 4, 2>(p, s, opt, blocks_out);
        return launch_gemv_cfg<WT, EPI, 2, 4, 1>(p, s, opt, blocks_out);
    }
    if constexpr (EPI == EPI_RESID && sizeof(WT) == 2) {
        if (p.part && ch <= 12) return launch_gemv_cfg<WT, EPI, 2, 4, 1>(p, s, opt, blocks_out);
        if (ch > 12 && ch <= 40) return launch_gemv_cfg<WT, EPI, 2, 4, 4>(p, s, opt, blocks_out);
    }
    if (ch <= 12) return launch_gemv_cfg<WT, EPI, 2, 2, 2>(p, s, opt, blocks_out);
    if (ch <= 40) return launch_gemv_cfg<WT, EPI, 4, 2, 4>(p, s, opt, blocks_out);
    return launch_gemv_cfg<WT, EPI, 4, 2, 8>(p, s, opt, blocks_out);
}

template <int EPI>
static hipError_t launch_gemv(const Dims& D, const GemvP& p, hipStream_t s, int* blocks_out = nullptr)
{
    if (D.wt == WT_BF16) return launch_gemv_t<uint16_t, EPI>(p, s, D.opt, blocks_out);
    if (D.wt == WT_F16) return launch_gemv_t<f16_t, EPI>(p, s, D.opt, blocks_out);
    return launch_gemv_t<float, EPI>(p, s, D.opt, blocks_out);
}

static void set_chain(GemvP& p, const Chain* ch)
{
    if (!ch) return;
    p.wait_flag = ch->wait_flag; p.wait_count = ch->wait_count; p.done_flag = ch->done_flag; p.gen = ch->gen; p.err = ch->err;
}

hipError_t gemv_qkv(const Dims& D, const void* wq, const void* wk, const void* wv, const float* gain, const float* x,
                    const float* rope, const int* pos_dev, int pos_off, float* qbuf, void* kc, void* vc, hipStream_t s,
                    const Chain* ch, int* blocks_out)
{
    if (D.hd > 128 || D.hd % 2) return hipErrorInvalidValue;   // the kernel stages one rotary row of hd floats in a 128-float LDS array
    GemvP p = {};
    set_chain(p, ch);
    p.w0 = wq; p.w1 = wk; p.w2 = wv; p.in = x; p.gain = gain; p.eps = D.eps; p.K = D.d;
    p.n_rows = D.dq + 2 * D.dkv;
    p.y = qbuf; p.kc = kc; p.vc = vc; p.kt = D.kt; p.rope = rope; p.pos_dev = pos_dev; p.pos_off = pos_off;
    p.hd = D.hd; p.dq = D.dq; p.dkv = D.dkv; p.max_seq = D.max_seq;
    return launch_gemv<EPI_QKV>(D, p, s, blocks_out);
}

hipError_t gemv_resid(const Dims& D, const void* w, int N, int K, const float* in, float* x, float* tap, hipStream_t s,
                      const Chain* ch, int* blocks_out)
{
    GemvP p = {};
    set_chain(p, ch);
    p.w0 = w; p.in = in; p.gain = nullptr; p.eps = D.eps; p.K = K; p.n_rows = N; p.y = x; p.tap = tap;
    return launch_gemv<EPI_RESID>(D, p, s, blocks_out);
}

hipError_t gemv_resid_attn(const Dims& D, const void* w, const float* part, int n_splits, float* x, float* tap,
                           hipStream_t s)
{
    if (n_splits < 1 || n_splits > GV_FOLD_MAX || D.hd % 4) return hipErrorInvalidValue;
    GemvP p = {};
    p.w0 = w; p.in = nullptr; p.part = part; p.n_splits = n_splits; p.hd = D.hd; p.gain = nullptr; p.eps = D.eps;
    p.K = D.dq; p.n_rows = D.d; p.y = x; p.tap = tap;
    return launch_gemv<EPI_RESID>(D, p, s);
}

hipError_t gemv_swiglu(const Dims& D, const void* wg, const void* wu, const float* gain, const float* x, float* act,
                       hipStream_t s, const Chain* ch, int* blocks_out)
{
    GemvP p = {};
    set_chain(p, ch);
    p.w0 = wg; p.w1 = wu; p.in = x; p.gain = gain; p.eps = D.eps; p.K = D.d; p.n_rows = 2 * D.f; p.y = act;
    return launch_gemv<EPI_SWIGLU>(D, p, s, blocks_out);
}

hipError_t gemv_lmhead(const Dims& D, const void* wlm, const float* gain, const float* x, float* logits, hipStream_t s)
{
    GemvP p = {};
    p.w0 = wlm; p.in = x; p.gain = gain; p.eps = D.eps; p.K = D.d; p.n_rows = D.V; p.y = logits;
    return launch_gemv<EPI_STORE>(D, p, s);
}

hipError_t gemv_lmhead_argmax(const Dims& D, const void* wlm, const float* gain, const float* x, float* logits, float clamp,
                              float* vstat, int32_t* tok_out, float* maxprob_out, hipStream_t s)
{
    if (!vstat) return hipErrorInvalidValue;
    GemvP p = {};
    p.w0 = wlm; p.in = x; p.gain = gain; p.eps = D.eps; p.K = D.d; p.n_rows = D.V; p.y = logits;
    p.vstat = vstat; p.clamp = clamp;
    int blocks = 0;
    hipError_t e = launch_gemv<EPI_STORE>(D, p, s, &blocks);
    if (e != hipSuccess) return e;
    if (blocks < 1 || blocks > GEMV_MAX_BLOCKS) return hipErrorInvalidValue;
    hipLaunchKernelGGL(vocab_finish_kernel, dim3(1), dim3(256), 0, s, vstat, blocks, tok_out, maxprob_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// multi-row path
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rmsnorm_rows_kernel(const float* __restrict__ in, const float* __restrict__ gain,
                                                           int K, float eps, float* __restrict__ out)
{
    __shared__ float red[4];
    const float* x = in + (size_t)blockIdx.x * K;
    float* o = out + (size_t)blockIdx.x * K;
    float ss = 0.f;
    for (int i = threadIdx.x * 4; i < K; i += 1024) {
        float4 v = *reinterpret_cast<const float4*>(x + i);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    float tot = block_sum<4>(ss, red);
    float sc = 1.0f / sqrtf(tot / (float)K + eps);
    for (int i = threadIdx.x * 4; i < K; i += 1024) {
        float4 v = *reinterpret_cast<const float4*>(x + i);
        float4 g = *reinterpret_cast<const float4*>(gain + i);
        v.x = v.x * sc * g.x; v.y = v.y * sc * g.y; v.z = v.z * sc * g.z; v.w = v.w * sc * g.w;
        *reinterpret_cast<float4*>(o + i) = v;
    }
}

hipError_t rmsnorm_rows(const float* in, const float* gain, int M, int K, float eps, float* out, hipStream_t s)
{
    hipLaunchKernelGGL(rmsnorm_rows_kernel, dim3(M), dim3(256), 0, s, in, gain, K, eps, out);
    return hipGetLastError();
}

struct RowsP {
    const void* w[3];
    int n[3];       // rows of each stacked matrix (multiples of 16)
    int K;
    const float* x; // [M][K]
    float* y; int ldy;
    float* tap; int tap_ld;
    int M;
};

enum { RM_STORE = 0, RM_RESID = 1, RM_SWIGLU = 2 };

__device__ __forceinline__ void rows_epilogue(const RowsP& p, int mode, int r, size_t col, float v, float v2)
{
    if (mode == RM_STORE) {
        p.y[(size_t)r * p.ldy + col] = v;
    } else if (mode == RM_RESID) {
        float* dst = p.y + (size_t)r * p.ldy + col;
        float t = *dst + v;
        *dst = t;
        if (p.tap) p.tap[(size_t)r * p.tap_ld + col] = t;
    } else {
        p.y[(size_t)r * p.ldy + col] = v / (1.0f + __expf(-v)) * v2;
    }
}

// --- bf16 weights: MFMA tiles -------------------------------------------------------------------
// One block owns 16 consecutive output rows (RM_SWIGLU: 16 gate rows and the matching 16 up rows).
// Its 8 waves interleave over the K dimension in steps of 32: the weight tile is the MFMA A
// operand loaded straight from global memory (lane (r, g): row r, 8 consecutive k at 8g), the
// activations are the B operand (lane (c, g): token row c, same 8 k), split on the fly into
// bf16 hi = rne(x) and lo = rne(x - hi), so that hi + lo carries 16 mantissa bits of x.
constexpr int MF_WAVES = 8;
constexpr int MF_THREADS = MF_WAVES * 64;

__device__ __forceinline__ void split_hi_lo(const float (&x)[8], bf16x8_t& hi, bf16x8_t& lo)
{
#pragma unroll
    for (int j = 0; j < 8; j++) {
        __bf16 h = (__bf16)x[j];
        hi[j] = h;
        lo[j] = (__bf16)(x[j] - (float)h);
    }
}

template <int MODE>
__global__ __launch_bounds__(MF_THREADS) void gemm_rows_mfma_kernel(RowsP p)
{
    __shared__ float red[MF_WAVES][2][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int K = p.K;

    // which matrix / row tile does this block own?
    int tile = blockIdx.x;
    const uint16_t* W0; const uint16_t* W1 = nullptr;
    size_t col0;  // first output column of the tile
    if (MODE == RM_SWIGLU) {
        W0 = (const uint16_t*)p.w[0] + (size_t)tile * 16 * K;
        W1 = (const uint16_t*)p.w[1] + (size_t)tile * 16 * K;
        col0 = (size_t)tile * 16;
    } else {
        int t0 = p.n[0] >> 4, t1 = p.n[1] >> 4;
        if (tile < t0) { W0 = (const uint16_t*)p.w[0] + (size_t)tile * 16 * K; col0 = (size_t)tile * 16; }
        else if (tile < t0 + t1) { W0 = (const uint16_t*)p.w[1] + (size_t)(tile - t0) * 16 * K; col0 = (size_t)tile * 16; }
        else { W0 = (const uint16_t*)p.w[2] + (size_t)(tile - t0 - t1) * 16 * K; col0 = (size_t)tile * 16; }
    }
    const uint16_t* a0p = W0 + (size_t)r16 * K + g * 8;
    const uint16_t* a1p = MODE == RM_SWIGLU ? W1 + (size_t)r16 * K + g * 8 : nullptr;
    const bool have_col = r16 < p.M;
    const float* bp = p.x + (size_t)(have_col ? r16 : 0) * K + g * 8;

    f32x4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    const int steps = (K + 31) >> 5;
#pragma unroll 2
    for (int st = wave; st < steps; st += MF_WAVES) {
        const int k0 = st << 5;
        const bool in_k = (k0 + g * 8) < K;  // K is a multiple of 8: a lane's 8 k are all in or all out
        bf16x8_t a0 = {}, a1 = {};
        float xb[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (in_k) {
            a0 = *reinterpret_cast<const bf16x8_t*>(a0p + k0);
            if (MODE == RM_SWIGLU) a1 = *reinterpret_cast<const bf16x8_t*>(a1p + k0);
            if (have_col) {
                float4 t0 = *reinterpret_cast<const float4*>(bp + k0);
                float4 t1 = *reinterpret_cast<const float4*>(bp + k0 + 4);
                xb[0] = t0.x; xb[1] = t0.y; xb[2] = t0.z; xb[3] = t0.w;
                xb[4] = t1.x; xb[5] = t1.y; xb[6] = t1.z; xb[7] = t1.w;
            }
        }
        bf16x8_t bh, bl;
        split_hi_lo(xb, bh, bl);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bh, acc0, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bl, acc0, 0, 0, 0);
        if (MODE == RM_SWIGLU) {
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bh, acc1, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bl, acc1, 0, 0, 0);
        }
    }
    // D layout: lane (c = lane % 16, g = lane / 16) holds rows 4g..4g+3 of column c
#pragma unroll
    for (int j = 0; j < 4; j++) {
        red[wave][0][(g * 4 + j) * 16 + r16] = acc0[j];
        if (MODE == RM_SWIGLU) red[wave][1][(g * 4 + j) * 16 + r16] = acc1[j];
    }
    __syncthreads();
    if (threadIdx.x < 256) {
        int row = threadIdx.x & 15;   // output feature within the tile (fastest: coalesced stores)
        int c = threadIdx.x >> 4;     // token row
        if (c < p.M) {
            float v = 0.f, v2 = 0.f;
#pragma unroll
            for (int w = 0; w < MF_WAVES; w++) {
                v += red[w][0][row * 16 + c];
                if (MODE == RM_SWIGLU) v2 += red[w][1][row * 16 + c];
            }
            rows_epilogue(p, MODE, c, col0 + row, v, v2);
        }
    }
}

// --- fp32 weights (and any dtype as a plain cross-check): FMA rows --------------------------------
// One wave owns 4 consecutive output rows (RM_SWIGLU: 2 gate + 2 up rows) and up to 4 token rows at a time.
template <typename WT, int MODE>
__global__ __launch_bounds__(256) void gemm_rows_fma_kernel(RowsP p)
{
    constexpr int VEC = Elem<WT>::VEC;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = p.K;
    const int n_out = MODE == RM_SWIGLU ? p.n[0] : p.n[0] + p.n[1] + p.n[2];
    const int n_units = MODE == RM_SWIGLU ? n_out / 2 : n_out / 4;
    for (int u = blockIdx.x * 4 + wave; u < n_units; u += gridDim.x * 4) {
        const WT* wr[4];
        size_t col[4];
        if (MODE == RM_SWIGLU) {
            size_t n = (size_t)u * 2;
            wr[0] = (const WT*)p.w[0] + n * K; wr[1] = (const WT*)p.w[1] + n * K;
            wr[2] = (const WT*)p.w[0] + (n + 1) * K; wr[3] = (const WT*)p.w[1] + (n + 1) * K;
            col[0] = n; col[1] = n; col[2] = n + 1; col[3] = n + 1;
        } else {
#pragma unroll
            for (int r = 0; r < 4; r++) {
                size_t n = (size_t)u * 4 + r;
                col[r] = n;
                if (n < (size_t)p.n[0]) wr[r] = (const WT*)p.w[0] + n * K;
                else if (n < (size_t)(p.n[0] + p.n[1])) wr[r] = (const WT*)p.w[1] + (n - p.n[0]) * K;
                else wr[r] = (const WT*)p.w[2] + (n - p.n[0] - p.n[1]) * K;
            }
        }
        for (int m0 = 0; m0 < p.M; m0 += 4) {
            float acc[4][4] = {};
            for (int k = lane * VEC; k < K; k += 64 * VEC) {
                float wv[4][VEC];
#pragma unroll
                for (int r = 0; r < 4; r++) Elem<WT>::load(wr[r] + k, wv[r]);
#pragma unroll
                for (int m = 0; m < 4; m++) {
                    if (m0 + m < p.M) {
                        const float* xr = p.x + (size_t)(m0 + m) * K + k;
#pragma unroll
                        for (int j = 0; j < VEC; j++) {
                            float xv = xr[j];
#pragma unroll
                            for (int r = 0; r < 4; r++) acc[r][m] = fmaf(wv[r][j], xv, acc[r][m]);
                        }
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; r++)
#pragma unroll
                for (int m = 0; m < 4; m++) acc[r][m] = wave_sum(acc[r][m]);
            if (lane == 0) {
                for (int m = 0; m < 4 && m0 + m < p.M; m++) {
                    if (MODE == RM_SWIGLU) {
                        rows_epilogue(p, MODE, m0 + m, col[0], acc[0][m], acc[1][m]);
                        rows_epilogue(p, MODE, m0 + m, col[2], acc[2][m], acc[3][m]);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; r++) rows_epilogue(p, MODE, m0 + m, col[r], acc[r][m], 0.f);
                    }
                }
            }
        }
    }
}

template <int MODE>
static hipError_t gemm_rows_mode(const Dims& D, const RowsP& p, hipStream_t s)
{
    if (D.wt == WT_BF16) {
        int tiles = MODE == RM_SWIGLU ? p.n[0] / 16 : (p.n[0] + p.n[1] + p.n[2]) / 16;
        hipLaunchKernelGGL((gemm_rows_mfma_kernel<MODE>), dim3(tiles), dim3(MF_THREADS), 0, s, p);
    } else {
        int n_out = MODE == RM_SWIGLU ? p.n[0] : p.n[0] + p.n[1] + p.n[2];
        int units = MODE == RM_SWIGLU ? n_out / 2 : n_out / 4;
        int blocks = ceil_div(units, 4);
        if (blocks > 4096) blocks = 4096;
        if (D.wt == WT_F16) hipLaunchKernelGGL((gemm_rows_fma_kernel<f16_t, MODE>), dim3(blocks), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((gemm_rows_fma_kernel<float, MODE>), dim3(blocks), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}

hipError_t gemm_rows(const Dims& D, const RowsGemm& g, hipStream_t s)
{
    RowsP p = {};
    for (int i = 0; i < 3; i++) { p.w[i] = g.w[i]; p.n[i] = g.n[i]; }
    p.K = g.K; p.x = g.x; p.y = g.y; p.ldy = g.ldy; p.tap = g.tap; p.tap_ld = g.tap_ld; p.M = g.M;
    if (g.M < 1 || g.M > 16) return hipErrorInvalidValue;
    switch (g.mode) {
        case RM_STORE: return gemm_rows_mode<RM_STORE>(D, p, s);
        case RM_RESID: return gemm_rows_mode<RM_RESID>(D, p, s);
        case RM_SWIGLU: return gemm_rows_mode<RM_SWIGLU>(D, p, s);
    }
    return hipErrorInvalidValue;
}

// --- bf16 weights, multi-row MFMA GEMM at streaming speed (K a multiple of 64) -----------------------
// The verify / prompt path.  Activations arrive already split into two bf16 arrays hi = rne(x),
// lo = rne(x - hi) (hi + lo carries 16 mantissa bits of x), written once by whoever produced x,
// so the GEMM itself is nothing but loads and MFMAs.  RMSNorm costs no kernel of its own: the
// projection that finishes a residual row block (RESID mode) also writes x * gain of the NEXT norm as
// hi/lo plus, per 16-column tile, the partial sums of x^2; the consumer adds the partials of a row,
// and scales its finished dot products by rsqrt(mean + eps) -- the scale is a per-row scalar and
// commutes with the contraction.
//   * QKV mode orders the 16 rows of a tile as 8 rotary pairs (i, i + hd/2), so the epilogue can
//     rotate q and k and write k, v straight into the cache; SwiGLU mode writes its result
//     directly as the hi/lo pair the down projection consumes.
constexpr int RM_QKV = 3;

struct RowsP2 {
    const void* w[3];
    int n[3];  // rows of each stacked matrix (multiples of 16); SWIGLU: n[0] = n[1] = f
    int K;
    const uint16_t* bh; const uint16_t* bl; int ldb;  // activations [M][ldb], bf16 hi and lo
    float* y; int ldy;                                // fp32 output (STORE / RESID / QKV: q)
    uint16_t* oh; uint16_t* ol; int ldo;              // SWIGLU: hi/lo output
    float* tap; int tap_ld;
    int M;
    const float* rope; const int* pos_dev; int pos_off;
    int hd, dq, dkv, max_seq;
    void* kc; void* vc; int kt;                 // cache rows of this layer, element type (WeightType code)
    const float* ssq; int n_ssq; float eps;     // consumer: partial sums of squares [M][n_ssq] of the input rows (or null)
    const float* gain_out; float* ssq_out;      // RESID producer: gain of the next norm -> oh/ol = split(x * gain), ssq_out [M][n/16]
    int ksplit; float* kpart;                   // wide RESID only: K cut into ksplit slices (grid.y), raw sums to kpart [ksplit][M][n]
    int tile0, fin_tile0;                       // large tiles: first weight tile of this launch; first 64-column output tile of its finishing launch
    int tap_only;                               // > 0: only row tap_only - 1 writes its tap (a prompt needs the last row's only)
    int n_tiles;                                // large-tile kernel: weight tiles of the launch
};

// hi = rne(v), lo = rne(v - hi) in the 16-bit storage type (bf16, or fp16 when f16 is set)
__device__ __forceinline__ void split_store(float v, uint16_t* hi, uint16_t* lo, size_t i, bool f16)
{
    const uint16_t h = f32_to_h16_bits(v, f16);
    hi[i] = h;
    lo[i] = f32_to_h16_bits(v - h16_bits_to_f32(h, f16), f16);
}
// 16x16x32 MFMA on two 128-bit operands holding 8 bf16 (or fp16) each
template <bool F16> __device__ __forceinline__ f32x4_t mfma_h16(u32x4_t a, u32x4_t b, f32x4_t c)
{
    if (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// weight row of logical row r16 of tile `tile`
template <int MODE>
__device__ __forceinline__ const uint16_t* m2_row(const RowsP2& p, int tile, int r16, int which /*SWIGLU: 0 gate, 1 up*/)
{
    if (MODE == RM_SWIGLU) return (const uint16_t*)p.w[which] + (size_t)(tile * 16 + r16) * p.K;
    if (MODE == RM_QKV) {
        const int tq = p.dq >> 4, tk = p.dkv >> 4;
        if (tile < tq + tk) {
            const uint16_t* base = (const uint16_t*)p.w[0];
            int tt = tile;
            if (tile >= tq) { base = (const uint16_t*)p.w[1]; tt = tile - tq; }
            const int tph = p.hd >> 4, head = tt / tph, th = tt % tph;
            const int row = head * p.hd + th * 8 + (r16 & 7) + (r16 >> 3) * (p.hd >> 1);
            return base + (size_t)row * p.K;
        }
        return (const uint16_t*)p.w[2] + (size_t)((tile - tq - tk) * 16 + r16) * p.K;
    }
    int row = tile * 16 + r16;
    if (row < p.n[0]) return (const uint16_t*)p.w[0] + (size_t)row * p.K;
    row -= p.n[0];
    if (row < p.n[1]) return (const uint16_t*)p.w[1] + (size_t)row * p.K;
    return (const uint16_t*)p.w[2] + (size_t)(row - p.n[1]) * p.K;
}

// v summed over the 16 lanes of a DPP row (rotations by 8, 4, 2, 1); every lane of the row gets the sum
template <int CTRL> __device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v)
{
    v = dpp_add<0x128>(v);  // row_ror:8
    v = dpp_add<0x124>(v);  // row_ror:4
    v = dpp_add<0x122>(v);  // row_ror:2
    return dpp_add<0x121>(v);  // row_ror:1
}
template <int CTRL> __device__ __forceinline__ float dpp_max(float v)
{
    return fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false)));
}
__device__ __forceinline__ float row16_max(float v)
{
    v = dpp_max<0x128>(v);
    v = dpp_max<0x124>(v);
    v = dpp_max<0x122>(v);
    return dpp_max<0x121>(v);
}

// Final step of a tile: sum the KS per-wave partial tiles held in LDS (layout [wave][NT][256], element
// row*16 + column) and apply the mode's epilogue.  Executed by the whole block (it contains barriers in QKV mode).
// rs: per-column (= activation row) RMS scale in LDS, 1 where no norm applies.
template <int MODE, bool F16>
__device__ __forceinline__ void m2_epilogue(const RowsP2& p, int t, const float* red, int KS, int ts, float* fin,
                                            const float* rs)
{
    constexpr int NT = MODE == RM_SWIGLU ? 2 : 1;
    const int tid = threadIdx.x;
    const int rr = tid & 15, c = (tid >> 4) & 15;
    float v = 0.f, v2 = 0.f;
    if (tid < 256) {
        for (int j = 0; j < KS; j++) {
            v += red[((ts * KS + j) * NT + 0) * 256 + rr * 16 + c];
            if (MODE == RM_SWIGLU) v2 += red[((ts * KS + j) * NT + 1) * 256 + rr * 16 + c];
        }
        if (MODE != RM_RESID) { v *= rs[c]; v2 *= rs[c]; }
        if (MODE == RM_QKV) fin[rr * 16 + c] = v;
    }
    if (MODE == RM_QKV) __syncthreads();
    if (tid < 256 && c < p.M) {
        if (MODE == RM_QKV) {
            const int tq = p.dq >> 4, tk = p.dkv >> 4;
            const int pos = p.pos_dev[0] + p.pos_off + c;
            if (t < tq + tk) {
                const bool is_q = t < tq;
                const int tt = is_q ? t : t - tq;
                const int tph = p.hd >> 4, head = tt / tph, th = tt % tph, half = p.hd >> 1;
                const int i = th * 8 + (rr & 7);
                const float av = fin[(rr & 7) * 16 + c], bv = fin[((rr & 7) + 8) * 16 + c];
                const float* cs = p.rope + ((size_t)pos * half + i) * 2;
                const float o = rr < 8 ? av * cs[0] - bv * cs[1] : bv * cs[0] + av * cs[1];
                const int e = rr < 8 ? i : i + half;
                if (is_q) p.y[(size_t)c * p.ldy + (size_t)head * p.hd + e] = o;
                else kv_put(p.kc, ((size_t)head * p.max_seq + pos) * p.hd + e, o, p.kt);
            } else {
                const int e = (t - tq - tk) * 16 + rr;
                kv_put(p.vc, ((size_t)(e / p.hd) * p.max_seq + pos) * p.hd + (e % p.hd), v, p.kt);
            }
        } else {
            const size_t colx = (size_t)t * 16 + rr;
            if (MODE == RM_STORE) p.y[(size_t)c * p.ldy + colx] = v;
            else if (MODE == RM_RESID) {
                float* dst = p.y + (size_t)c * p.ldy + colx;
                const float tv = *dst + v;
                *dst = tv;
                if (p.tap) p.tap[(size_t)c * p.tap_ld + colx] = tv;
                if (p.gain_out) {
                    split_store(tv * p.gain_out[colx], p.oh, p.ol, (size_t)c * p.ldo + colx, F16);
                    // the 16 threads of one column are the 16 lanes of a DPP row, all active together
                    const float sq = row16_sum(tv * tv);
                    if (rr == 0) p.ssq_out[(size_t)c * (p.n[0] >> 4) + t] = sq;
                }
            } else split_store(v / (1.0f + __expf(-v)) * v2, p.oh, p.ol, (size_t)c * p.ldo + colx, F16);
        }
    }
    if (MODE == RM_QKV) __syncthreads();
}

// LDS-staged variant: the block fetches a 16-row x 512-k stripe of the weights the way the single-row
// GEMV does -- every wave two whole rows, 1 KB contiguous per load instruction, which is the access
// shape that streams fastest from HBM -- plus the matching slice of the hi/lo activations, parks both
// in LDS, and the MFMA operands are then read from LDS in fragment order.  Activations never enter
// the in-order global-load queue between weight loads, so the next stripe's loads stay in flight
// during the whole MFMA phase.
constexpr int M3_CK = 512;
constexpr int M3_PITCH = M3_CK * 2 + 16;  // bytes per LDS row (16-byte pad spreads the banks)

// M3_D = stripes in flight per block; F16: fp16 storage, else bf16; NU = activation vectors per thread and stripe
// (2 covers up to 8 rows, 3 up to 12, 4 up to 16)
template <int MODE, int M3_D, bool F16, int NU>
__global__ __launch_bounds__(512, (NU <= 2 ? 6 : NU == 3 ? 5 : 4)) void rows_mfma3_kernel(RowsP2 p)
{
    constexpr int NT = MODE == RM_SWIGLU ? 2 : 1;
    extern __shared__ __align__(16) unsigned char sm3[];
    __shared__ float fin[256];
    __shared__ float rs[16];
    unsigned char* As = sm3;                          // [NT][16][PITCH]
    unsigned char* Bh = sm3 + NT * 16 * M3_PITCH;     // [M][PITCH]
    unsigned char* Bl = Bh + p.M * M3_PITCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int tile = blockIdx.x;
    const int K = p.K, M = p.M;
    const int NC = (K + M3_CK - 1) / M3_CK;

    const uint16_t* ap[NT][2];
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
        for (int j = 0; j < 2; j++) ap[t][j] = m2_row<MODE>(p, tile, 2 * wave + j, t);
    // activation vectors (16 bytes each) of one stripe: [hi|lo][M][64]; thread takes v = tid, tid+512, ...
    const int nbv = M * 128;
    const uint16_t* bsrc[NU];
    int bdst[NU];
    int bk[NU];
#pragma unroll
    for (int u = 0; u < NU; u++) {
        const int v = min(tid + u * 512, nbv - 1);
        const int which = v / (M * 64), rem = v % (M * 64), c = rem >> 6, kk = (rem & 63) * 8;
        bsrc[u] = (which ? p.bl : p.bh) + (size_t)c * p.ldb;
        bdst[u] = (which ? M : 0) * M3_PITCH + c * M3_PITCH + kk * 2;
        bk[u] = kk;
    }
    // Register ring: the loads of the next M3_D stripes are in flight while one stripe is multiplied.  Every load is
    // UNCONDITIONAL: addresses past the end of K (or past the last activation vector) are clamped to valid ones and
    // the values are replaced by zeros when the stripe is stored to LDS.  With loads under conditions the compiler
    // cannot count what is in flight and waits for everything, the stripes just requested included.
    u32x4_t ra[M3_D][NT][2], rb[M3_D][NU];
    const u32x4_t zero4 = {0u, 0u, 0u, 0u};
    auto gload = [&](int slot, int ck) {
        const int k0 = ck * M3_CK;
        const int ka = min(k0 + lane * 8, K - 8);
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int j = 0; j < 2; j++) ra[slot][t][j] = gv_load(ap[t][j] + ka);
#pragma unroll
        for (int u = 0; u < NU; u++) rb[slot][u] = *reinterpret_cast<const u32x4_t*>(bsrc[u] + min(k0 + bk[u], K - 8));
    };
    f32x4_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; t++) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int bc = min(r16, M - 1);  // columns >= M read a valid row; their results are never stored
    auto stage = [&](int slot, int ck) {
        const int k0 = ck * M3_CK;
        const bool ok = k0 + lane * 8 < K;
        __syncthreads();  // previous stripe fully consumed
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int j = 0; j < 2; j++)
                *reinterpret_cast<u32x4_t*>(As + (t * 16 + 2 * wave + j) * M3_PITCH + lane * 16) = ok ? ra[slot][t][j] : zero4;
#pragma unroll
        for (int u = 0; u < NU; u++)
            if (tid + u * 512 < nbv) *reinterpret_cast<u32x4_t*>(Bh + bdst[u]) = k0 + bk[u] < K ? rb[slot][u] : zero4;
        __syncthreads();
    };
    auto multiply = [&](int ck) {
        const int nks = min(M3_CK / 32, (K - ck * M3_CK) / 32);
        for (int s = wave; s < nks; s += 8) {
            const int off = s * 64 + g * 16;
            const u32x4_t bh = *reinterpret_cast<const u32x4_t*>(Bh + bc * M3_PITCH + off);
            const u32x4_t bl = *reinterpret_cast<const u32x4_t*>(Bl + bc * M3_PITCH + off);
#pragma unroll
            for (int t = 0; t < NT; t++) {
                const u32x4_t w = *reinterpret_cast<const u32x4_t*>(As + (t * 16 + r16) * M3_PITCH + off);
                acc[t] = mfma_h16<F16>(w, bh, acc[t]);
                acc[t] = mfma_h16<F16>(w, bl, acc[t]);
            }
        }
    };
    // The blocks of a launch start together and would all ask the memory channels for the same stripe at the same time:
    // block `tile` starts its walk over K at stripe (tile / 8) % NC and wraps around (workgroups go to the eight XCDs
    // round-robin by id, so blocks that follow each other on one XCD start one stripe apart).  Measured against a walk
    // from 0 in every block: 7B QKV 28.0 -> 25.1 us, gate/up 39.4 -> 36.3, down 24.6 -> 22.6; 70B gate/up 170 -> 147,
    // output projection 35 -> 29, LM head 108 -> 90 (a start at tile % NC instead is 20 % SLOWER than a walk from 0 at
    // K = 8192).
    const int rot = (tile / 8) % NC;
    auto sidx = [&](int i) { const int c = min(i, NC - 1) + rot; return c >= NC ? c - NC : c; };
#pragma unroll
    for (int sl = 0; sl < M3_D; sl++) gload(sl, sidx(sl));
    // RMS scale of every activation row from the producer's per-tile sums of squares (read by the epilogue).
    // Measured per mode: gate/up (long-lived blocks, two stripes in flight) loses least when the partials are
    // summed after the weight stream, the short-lived blocks of QKV and the LM head when it happens up front.
    auto row_scales = [&]() {
        for (int c = wave; c < M; c += 8) {
            float sq = 0.f;
            for (int i = lane; i < p.n_ssq; i += 64) sq += p.ssq[(size_t)c * p.n_ssq + i];
            sq = wave_sum(sq);
            if (lane == 0) rs[c] = 1.0f / sqrtf(sq / (float)K + p.eps);
        }
    };
    if (tid < 16) rs[tid] = 1.0f;
    if (MODE != RM_RESID && MODE != RM_SWIGLU && p.ssq) row_scales();
    // steady state: every step stores its slot's stripe, refills the slot and multiplies; the stripe count is padded
    // to a multiple of M3_D (a padding request re-reads the last stripe and is never stored); the last M3_D steps
    // request nothing
    const int NCp = (NC + M3_D - 1) / M3_D * M3_D;
    int ck0 = 0;
    for (; ck0 + M3_D < NCp; ck0 += M3_D) {
#pragma unroll
        for (int sl = 0; sl < M3_D; sl++) {
            stage(sl, sidx(ck0 + sl));
            gload(sl, sidx(ck0 + sl + M3_D));
            multiply(sidx(ck0 + sl));
        }
    }
#pragma unroll
    for (int sl = 0; sl < M3_D; sl++) {
        if (ck0 + sl < NC) {   // uniform
            stage(sl, sidx(ck0 + sl));
            multiply(sidx(ck0 + sl));
        }
    }
    if (MODE == RM_SWIGLU && p.ssq) row_scales();
    __syncthreads();
    float* red = reinterpret_cast<float*>(sm3);  // [8][NT][256] floats fit inside the weight stripe area
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
        for (int j = 0; j < 4; j++) red[(wave * NT + t) * 256 + (g * 4 + j) * 16 + r16] = acc[t][j];
    __syncthreads();
    m2_epilogue<MODE, F16>(p, tile, red, 8, 0, fin, rs);
}

template <int MODE, int DEPTH, bool F16, int NU>
static hipError_t launch_mfma3_nu(const RowsP2& p, int n_tiles, hipStream_t s)
{
    constexpr int NT = MODE == RM_SWIGLU ? 2 : 1;
    const size_t lds = (size_t)(NT * 16 + 2 * p.M) * M3_PITCH;
    static std::atomic<size_t> lds_limit{0};  // per instantiation
    {
        hipError_t e = ensure_lds((const void*)rows_mfma3_kernel<MODE, DEPTH, F16, NU>, lds, lds_limit);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((rows_mfma3_kernel<MODE, DEPTH, F16, NU>), dim3(n_tiles), dim3(512), lds, s, p);
    return hipGetLastError();
}

template <int MODE, int DEPTH, bool F16>
static hipError_t launch_mfma3(const RowsP2& p, int n_tiles, hipStream_t s)
{
    if (p.M <= 8) return launch_mfma3_nu<MODE, DEPTH, F16, 2>(p, n_tiles, s);
    if (p.M <= 12) return launch_mfma3_nu<MODE, DEPTH, F16, 3>(p, n_tiles, s);
    return launch_mfma3_nu<MODE, DEPTH, F16, 4>(p, n_tiles, s);
}

template <int MODE, bool F16>
static hipError_t rows_fused_mode(const RowsP2& p, hipStream_t s, const LaunchOpts* opt)
{
    const int forced = opt ? opt->rows_depth : 0;
    const int n_tiles = MODE == RM_SWIGLU ? p.n[0] / 16 : (p.n[0] + p.n[1] + p.n[2]) / 16;
    // measured (`KB_ROWS=1 kernel_bench`, and at the 13B / 70B / Llama-3-8B shapes): two stripes in flight are best or
    // equal everywhere except gate/up, whose ring for two stripes of two matrices does not fit the registers of three
    // blocks per CU (the kernel is compiled for six waves per SIMD)
    const int depth = forced > 0 ? forced : (MODE == RM_SWIGLU ? 1 : 2);
    switch (depth) {
        case 1: return launch_mfma3<MODE, 1, F16>(p, n_tiles, s);
        case 2: return launch_mfma3<MODE, 2, F16>(p, n_tiles, s);
        default: return launch_mfma3<MODE, 3, F16>(p, n_tiles, s);
    }
}

// --- wide-block variant: up to 64 activation rows per pass (prompt blocks, the 2L confidence rows) -------
// With that many rows a 16-row weight tile would pull eight times more activation bytes out of the cache
// than weight bytes out of HBM.  Here a block owns 64 weight rows (64 of each matrix in SwiGLU mode) and all
// (<= 64) rows.  64 x 128-k stripes of the weights (non-temporal) and of the hi/lo rows go through LDS; a
// stripe has four 32-wide k-steps: wave w takes k-step w & 3 for the weight rows 32 (w >> 2) .. +31 and all
// rows, so every staged byte is read twice only, and the four k-step partials are summed through LDS at the
// end, band by band of 16 rows, where the mode's epilogue is applied.  52 KB of LDS per block (70 KB for
// SwiGLU): two to three blocks share a CU and cover each other's load / stage / multiply phases, which
// measured better than a deeper register ring.  Same modes, same RMSNorm folding and the same rotary-pair
// row order (here 32 pairs per tile) as the 16-row kernel.
constexpr int M6_CK = 128;
constexpr int M6_PITCH = M6_CK * 2 + 16;

// weight row of logical row r64 of tile `tile`
template <int MODE>
__device__ __forceinline__ const uint16_t* m6_row(const RowsP2& p, int tile, int r64, int which /*SWIGLU: 0 gate, 1 up*/)
{
    if (MODE == RM_SWIGLU) return (const uint16_t*)p.w[which] + (size_t)(tile * 64 + r64) * p.K;
    if (MODE == RM_QKV) {
        const int tq = p.dq >> 6, tk = p.dkv >> 6;
        if (tile < tq + tk) {
            const uint16_t* base = (const uint16_t*)p.w[0];
            int tt = tile;
            if (tile >= tq) { base = (const uint16_t*)p.w[1]; tt = tile - tq; }
            const int tph = p.hd >> 6, head = tt / tph, th = tt % tph;
            const int row = head * p.hd + th * 32 + (r64 & 31) + (r64 >> 5) * (p.hd >> 1);
            return base + (size_t)row * p.K;
        }
        return (const uint16_t*)p.w[2] + (size_t)((tile - tq - tk) * 64 + r64) * p.K;
    }
    int row = tile * 64 + r64;
    if (row < p.n[0]) return (const uint16_t*)p.w[0] + (size_t)row * p.K;
    row -= p.n[0];
    if (row < p.n[1]) return (const uint16_t*)p.w[1] + (size_t)row * p.K;
    return (const uint16_t*)p.w[2] + (size_t)(row - p.n[1]) * p.K;
}

// Epilogue of one output of the 64-row tiling: activation row m, weight row nn (= lane: a wave holds the 64
// weight rows of tile `tile` for one m) with finished, scaled sums v (and v2 of the second matrix in SwiGLU mode).
// Called by whole waves with m uniform (the RESID branch reduces over the wave, the QKV branch exchanges the two
// rows of a rotary pair, nn and nn ^ 32, by a shuffle).
template <int MODE, bool F16>
__device__ __forceinline__ void m6_epilogue(const RowsP2& p, int tile, int m, int nn, float v, float v2)
{
    const size_t colx = (size_t)tile * 64 + nn;
    if (MODE == RM_STORE) {
        p.y[(size_t)m * p.ldy + colx] = v;
    } else if (MODE == RM_SWIGLU) {
        split_store(v / (1.0f + __expf(-v)) * v2, p.oh, p.ol, (size_t)m * p.ldo + colx, F16);
    } else if (MODE == RM_RESID) {
        float* dst = p.y + (size_t)m * p.ldy + colx;
        const float tv = *dst + v;
        *dst = tv;
        if (p.tap && (p.tap_only <= 0 || m == p.tap_only - 1)) p.tap[(size_t)(p.tap_only > 0 ? 0 : m) * p.tap_ld + colx] = tv;
        if (p.gain_out) {
            split_store(tv * p.gain_out[colx], p.oh, p.ol, (size_t)m * p.ldo + colx, F16);
            const float sq = wave_sum(tv * tv);   // the wave holds the tile's 64 columns of row m
            if (nn == 0) p.ssq_out[(size_t)m * (p.n[0] >> 6) + tile] = sq;
        }
    } else {  // QKV: rotary pairs are (nn, nn + 32) for nn < 32
        const int tq = p.dq >> 6, tk = p.dkv >> 6;
        const int pos = p.pos_dev[0] + p.pos_off + m;
        const float other = __shfl_xor(v, 32, 64);
        if (tile < tq + tk) {
            const bool is_q = tile < tq;
            const int tt = is_q ? tile : tile - tq;
            const int tph = p.hd >> 6, head = tt / tph, th = tt % tph, half = p.hd >> 1;
            const int i = th * 32 + (nn & 31);
            const float av = nn < 32 ? v : other, bv = nn < 32 ? other : v;
            const float* cs = p.rope + ((size_t)pos * half + i) * 2;
            const float ov = nn < 32 ? av * cs[0] - bv * cs[1] : bv * cs[0] + av * cs[1];
            const int e = nn < 32 ? i : i + half;
            if (is_q) p.y[(size_t)m * p.ldy + (size_t)head * p.hd + e] = ov;
            else kv_put(p.kc, ((size_t)head * p.max_seq + pos) * p.hd + e, ov, p.kt);
        } else {
            const int e = (tile - tq - tk) * 64 + nn;
            kv_put(p.vc, ((size_t)(e / p.hd) * p.max_seq + pos) * p.hd + (e % p.hd), v, p.kt);
        }
    }
}

template <int MODE, bool F16, int M6_D>  // M6_D = stripes in flight per block
__global__ __launch_bounds__(512) void rows_wide_kernel(RowsP2 p)
{
    constexpr int NT = MODE == RM_SWIGLU ? 2 : 1;
    extern __shared__ __align__(16) unsigned char sm6[];
    __shared__ float rs[64];
    unsigned char* As = sm6;                            // [NT * 64][PITCH]
    unsigned char* Bh = sm6 + NT * 64 * M6_PITCH;       // [64][PITCH]
    unsigned char* Bl = Bh + 64 * M6_PITCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int tile = blockIdx.x, n0 = tile * 64;
    const int K = p.K, M = p.M;
    // this block's stripes: all of K, or slice blockIdx.y of ksplit (projections with few tiles are cut along K so
    // that every CU has a block; their raw sums go to kpart and rows_finish_resid_kernel adds them up in order)
    const int NCall = K / M6_CK;
    const int S = p.ksplit > 1 ? p.ksplit : 1;
    const int c_begin = (int)((long)NCall * blockIdx.y / S), NC = (int)((long)NCall * (blockIdx.y + 1) / S) - c_begin;
    // weights: wave w loads logical rows 8w .. 8w+7; instruction j covers rows 8w+4j .. 8w+4j+3 (16 lanes = 256 B per row)
    const int arow = 8 * wave + (lane >> 4), acol = (lane & 15) * 8;
    const uint16_t* ap[NT][2];
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
        for (int j = 0; j < 2; j++) ap[t][j] = m6_row<MODE>(p, tile, arow + 4 * j, t) + acol;
    // activations: 64 rows x 16 vectors per array; thread takes vectors tid and tid + 512 (row clamped to M - 1)
    const uint16_t* bhp[2];
    const uint16_t* blp[2];
    int bdst[2];
#pragma unroll
    for (int u = 0; u < 2; u++) {
        const int v = tid + u * 512, row = v >> 4, kk = (v & 15) * 8;
        const size_t off = (size_t)min(row, M - 1) * p.ldb + kk;
        bhp[u] = p.bh + off; blp[u] = p.bl + off;
        bdst[u] = row * M6_PITCH + kk * 2;
    }
    u32x4_t ra[M6_D][NT][2], rh[M6_D][2], rl[M6_D][2];
    auto gload = [&](int slot, int ck) {
        const int k0 = (c_begin + ck) * M6_CK;
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int j = 0; j < 2; j++) ra[slot][t][j] = gv_load(ap[t][j] + k0);
#pragma unroll
        for (int u = 0; u < 2; u++) {
            rh[slot][u] = *reinterpret_cast<const u32x4_t*>(bhp[u] + k0);
            rl[slot][u] = *reinterpret_cast<const u32x4_t*>(blp[u] + k0);
        }
    };
    auto stage = [&](int slot) {
        __syncthreads();
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int j = 0; j < 2; j++)
                *reinterpret_cast<u32x4_t*>(As + (t * 64 + arow + 4 * j) * M6_PITCH + acol * 2) = ra[slot][t][j];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            *reinterpret_cast<u32x4_t*>(Bh + bdst[u]) = rh[slot][u];
            *reinterpret_cast<u32x4_t*>(Bl + bdst[u]) = rl[slot][u];
        }
        __syncthreads();
    };
    const int kq = wave & 3, nh = wave >> 2;             // k-step of the stripe, half of the weight rows
    const int MT = (M + 15) >> 4;                        // live 16-row groups of activation rows
    f32x4_t acc[NT][2][4];
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) acc[t][i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    auto multiply = [&]() {
        const int off = kq * 64 + g * 16;
        u32x4_t a[NT][2];
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int i = 0; i < 2; i++)
                a[t][i] = *reinterpret_cast<const u32x4_t*>(As + (t * 64 + (nh * 2 + i) * 16 + r16) * M6_PITCH + off);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if (j < MT) {   // uniform
                const u32x4_t h = *reinterpret_cast<const u32x4_t*>(Bh + (j * 16 + r16) * M6_PITCH + off);
                const u32x4_t l = *reinterpret_cast<const u32x4_t*>(Bl + (j * 16 + r16) * M6_PITCH + off);
                // independent accumulators between the two updates of any one of them
#pragma unroll
                for (int t = 0; t < NT; t++)
#pragma unroll
                    for (int i = 0; i < 2; i++) acc[t][i][j] = mfma_h16<F16>(a[t][i], h, acc[t][i][j]);
#pragma unroll
                for (int t = 0; t < NT; t++)
#pragma unroll
                    for (int i = 0; i < 2; i++) acc[t][i][j] = mfma_h16<F16>(a[t][i], l, acc[t][i][j]);
            }
        }
    };
#pragma unroll
    for (int sl = 0; sl < M6_D; sl++)
        if (sl < NC) gload(sl, sl);
    // RMS scale of every activation row from the producer's per-tile sums of squares (read by the epilogue)
    if (tid < 64) rs[tid] = 1.0f;
    if (MODE != RM_RESID && p.ssq && S == 1) {   // (a K-split launch leaves the scaling to its finishing kernel)
        __syncthreads();
        for (int c = wave; c < M; c += 8) {
            float sq = 0.f;
            for (int i = lane; i < p.n_ssq; i += 64) sq += p.ssq[(size_t)c * p.n_ssq + i];
            sq = wave_sum(sq);
            if (lane == 0) rs[c] = 1.0f / sqrtf(sq / (float)K + p.eps);
        }
    }
    int ck0 = 0;
    for (; ck0 + 2 * M6_D <= NC; ck0 += M6_D) {   // steady state: every step refills its slot
#pragma unroll
        for (int sl = 0; sl < M6_D; sl++) {
            stage(sl);
            gload(sl, ck0 + sl + M6_D);
            multiply();
        }
    }
    for (; ck0 < NC; ck0 += M6_D) {               // drain
#pragma unroll
        for (int sl = 0; sl < M6_D; sl++) {
            if (ck0 + sl < NC) {
                stage(sl);
                if (ck0 + sl + M6_D < NC) gload(sl, ck0 + sl + M6_D);
                multiply();
            }
        }
    }
    // Sum the four k-step partials of every output, one band of 16 activation rows at a time, through LDS:
    // red[t][wave][i][256], element row * 16 + column of the D layout (lane (c = lane % 16, g) holds weight
    // rows 4g .. 4g+3 of activation row c), then the epilogue: thread -> (weight row nn, activation row c).
    float* red = reinterpret_cast<float*>(sm6);   // NT x 8 x 2 x 256 floats = NT x 16 KB
    for (int j = 0; j < MT; j++) {
        __syncthreads();
#pragma unroll
        for (int t = 0; t < NT; t++)
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    float v;
                    switch (j) {  // acc is indexed by compile-time constants only
                        case 0: v = acc[t][i][0][e]; break;
                        case 1: v = acc[t][i][1][e]; break;
                        case 2: v = acc[t][i][2][e]; break;
                        default: v = acc[t][i][3][e]; break;
                    }
                    red[((t * 8 + wave) * 2 + i) * 256 + (g * 4 + e) * 16 + r16] = v;
                }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 2; it++) {   // 64 weight rows x 16 activation rows = 1024 outputs, two per thread
            const int o = tid + it * 512;
            const int nn = o & 63, c = o >> 6;      // c (and so m) is uniform over a wave, nn = lane
            const int st = nn >> 4, hh = st >> 1, ii = st & 1;
            float v = 0.f, v2 = 0.f;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                v += red[((hh * 4 + q) * 2 + ii) * 256 + (nn & 15) * 16 + c];
                if (MODE == RM_SWIGLU) v2 += red[(((8 + hh * 4 + q) * 2) + ii) * 256 + (nn & 15) * 16 + c];
            }
            const int m = j * 16 + c;
            if (m >= M) continue;
            if (S > 1) {   // raw sums of this K slice: [slice][matrix][M][n_total]
                const size_t nt = (size_t)gridDim.x * 64;
                p.kpart[(((size_t)blockIdx.y * NT + 0) * M + m) * nt + n0 + nn] = v;
                if (MODE == RM_SWIGLU) p.kpart[(((size_t)blockIdx.y * NT + 1) * M + m) * nt + n0 + nn] = v2;
                continue;
            }
            if (MODE != RM_RESID) { v *= rs[m]; v2 *= rs[m]; }
            m6_epilogue<MODE, F16>(p, tile, m, nn, v, v2);
        }
    }
}

// Second half of a K-split launch: one wave per (FIN_ROWS rows, 64-column tile) adds the slices in a fixed order,
// applies the RMS scale of each row (summing the producer's partials itself) and runs the mode's epilogue.  The
// loads of the wave's rows are independent and issued together.
constexpr int FIN_ROWS = 4;
template <int MODE, bool F16>
__global__ __launch_bounds__(64) void rows_finish_kernel(RowsP2 p)
{
    constexpr int NT = MODE == RM_SWIGLU ? 2 : 1;
    const int tile = blockIdx.x + p.fin_tile0, lane = threadIdx.x;   // kpart covers this launch's tiles only
    const int mbase = blockIdx.y * FIN_ROWS;
    const size_t nt = (size_t)gridDim.x * 64, colx = (size_t)blockIdx.x * 64 + lane;
    float v[FIN_ROWS], v2[FIN_ROWS];
#pragma unroll
    for (int r = 0; r < FIN_ROWS; r++) v[r] = v2[r] = 0.f;
    for (int sl = 0; sl < p.ksplit; sl++) {
#pragma unroll
        for (int r = 0; r < FIN_ROWS; r++) {
            const int m = min(mbase + r, p.M - 1);   // rows past M re-read the last row, never written
            v[r] += p.kpart[(((size_t)sl * NT + 0) * p.M + m) * nt + colx];
            if (MODE == RM_SWIGLU) v2[r] += p.kpart[(((size_t)sl * NT + 1) * p.M + m) * nt + colx];
        }
    }
#pragma unroll
    for (int r = 0; r < FIN_ROWS; r++) {
        const int m = mbase + r;
        if (m >= p.M) break;   // uniform
        float a = v[r], b = v2[r];
        if (MODE != RM_RESID && p.ssq) {
            float sq = 0.f;
            for (int i = lane; i < p.n_ssq; i += 64) sq += p.ssq[(size_t)m * p.n_ssq + i];
            const float sc = 1.0f / sqrtf(wave_sum(sq) / (float)p.K + p.eps);
            a *= sc; b *= sc;
        }
        m6_epilogue<MODE, F16>(p, tile, m, lane, a, b);
    }
}

// --- large-tile variant: any number of activation rows in one launch (whole prompts, the context window) --------
// With hundreds of rows the work is a real GEMM and the weights should cross the chip once, not once per 64 rows.
// A block owns TN logical weight rows (TN / 2 gate + TN / 2 up rows in SwiGLU mode) x 128 activation rows; the blocks
// that share a weight tile run back to back on one XCD and all but the first find it in that L2.  64-wide K stripes of
// the weights and of the hi / lo rows go through LDS (register prefetch two stripes ahead; TN = 256 keeps two staging
// buffers and writes the next stripe while one is multiplied); the waves form a (TN / 64) x 2 grid of 64 x 64
// sub-tiles, 32 MFMAs (hi and lo) per 12 LDS fragment reads.  The finished tile goes back through LDS in two halves
// so that the epilogue sees (row, TN consecutive columns): same modes, same RMSNorm folding as the 64-row kernel;
// weight rows in natural order (a rotary pair e, e + hd/2 sits in one tile).
constexpr int MB_TM = 128, MB_CK = 64;
constexpr int MB_PITCH = MB_CK * 2 + 16;   // bytes per staged row

// weight row of logical row r of tile `tile` (TN logical rows per tile; SwiGLU: TN/2 gate rows, then TN/2 up rows)
template <int MODE, int TN>
__device__ __forceinline__ const uint16_t* mb_row(const RowsP2& p, int tile, int r)
{
    if (MODE == RM_SWIGLU) return (const uint16_t*)p.w[r / (TN / 2)] + (size_t)(tile * (TN / 2) + r % (TN / 2)) * p.K;
    int row = tile * TN + r;
    if (row < p.n[0]) return (const uint16_t*)p.w[0] + (size_t)row * p.K;
    row -= p.n[0];
    if (row < p.n[1]) return (const uint16_t*)p.w[1] + (size_t)row * p.K;
    return (const uint16_t*)p.w[2] + (size_t)(row - p.n[1]) * p.K;
}

// TN = weight rows per tile: 128 (256 threads, two blocks per CU) or 256 (512 threads, one block per CU: a third
// fewer bytes per MFMA through the CU's memory path, which is what bounds this kernel; used when the launch still
// has blocks for most CUs)
template <int MODE, bool F16, int TN>
__global__ __launch_bounds__(TN * 2, 2) void rows_big_kernel(RowsP2 p)
{
    constexpr int NTH = TN * 2, WN = TN / 64;   // threads; waves along the weight rows (x 2 along the activation rows)
    constexpr int RPS = NTH / 8;                // rows covered by one load step of the block
    constexpr int BU = MB_TM / RPS;             // load steps per activation plane
    constexpr int EP = TN + 4;                  // floats per row of the epilogue tile
    constexpr int NBUF = TN == 256 ? 2 : 1;     // staging buffers: the large tile (one block per CU) double-buffers in LDS
    constexpr int BUFB = (TN + 2 * MB_TM) * MB_PITCH;
    extern __shared__ __align__(16) unsigned char smb[];
    __shared__ float rs[MB_TM];
    unsigned char* Ws = smb;                          // [TN][PITCH]
    unsigned char* Bh = smb + TN * MB_PITCH;          // [128][PITCH]
    unsigned char* Bl = Bh + MB_TM * MB_PITCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int K = p.K, M = p.M;
    const int NCall = K / MB_CK;
    const int S = p.ksplit > 1 ? p.ksplit : 1;
    // Block id -> (weight tile and K slice, row block).  Workgroups go to the eight XCDs round-robin by id and each
    // XCD has its own L2: ids c, c + 8, c + 16, .. (one XCD, dispatched back to back) take the row blocks of ONE
    // weight tile, so the tile comes out of HBM once per XCD and the other row blocks find it in that L2.
    int tile, slice, m0;
    {
        const int mb = (M + MB_TM - 1) / MB_TM, units = p.n_tiles * S;
        const int L = blockIdx.x, full = units & ~7;
        int unit, y;
        if (L < full * mb) { const int ch = L / (8 * mb), r = L % (8 * mb); unit = ch * 8 + (r & 7); y = r >> 3; }
        else { const int r = L - full * mb, rem = units - full; unit = full + r % rem; y = r / rem; }
        tile = p.tile0 + unit % p.n_tiles; slice = unit / p.n_tiles; m0 = y * MB_TM;
    }
    const int c_begin = (int)((long)NCall * slice / S), NC = (int)((long)NCall * (slice + 1) / S) - c_begin;
    // a stripe is TN + 2 x 128 rows of 8 vectors of 16 bytes; thread takes row tid / 8 + RPS u, vector tid % 8.
    // Addresses are a block-uniform base plus a 32-bit element offset per thread (few registers: two stripes are in
    // flight per thread).
    const int kk = (tid & 7) * 8;
    const uint16_t* wb[4];   // uniform over the block
    int boff[BU], dstb[BU];
    const int woff = (tid >> 3) * K + kk, dstw = (tid >> 3) * MB_PITCH + kk * 2;
#pragma unroll
    for (int u = 0; u < 4; u++) wb[u] = mb_row<MODE, TN>(p, tile, RPS * u);
#pragma unroll
    for (int u = 0; u < BU; u++) {
        const int row = (tid >> 3) + RPS * u;
        boff[u] = min(m0 + row, M - 1) * p.ldb + kk;   // rows past M read a valid row, never stored
        dstb[u] = row * MB_PITCH + kk * 2;
    }
    constexpr int MB_D = 2;   // stripes in flight
    u32x4_t rw[MB_D][4], rh[MB_D][BU], rl[MB_D][BU];
    auto gload = [&](int slot, int ck) {
        const int k0 = (c_begin + ck) * MB_CK;
#pragma unroll
        for (int u = 0; u < 4; u++)   // cached loads: the other row blocks read the same tile
            rw[slot][u] = *reinterpret_cast<const u32x4_t*>(wb[u] + woff + k0);
#pragma unroll
        for (int u = 0; u < BU; u++) {
            rh[slot][u] = *reinterpret_cast<const u32x4_t*>(p.bh + boff[u] + k0);
            rl[slot][u] = *reinterpret_cast<const u32x4_t*>(p.bl + boff[u] + k0);
        }
    };
    auto put = [&](int slot, int buf) {   // registers of `slot` -> staging buffer `buf`
#pragma unroll
        for (int u = 0; u < 4; u++) *reinterpret_cast<u32x4_t*>(Ws + buf * BUFB + dstw + u * RPS * MB_PITCH) = rw[slot][u];
#pragma unroll
        for (int u = 0; u < BU; u++) {
            *reinterpret_cast<u32x4_t*>(Bh + buf * BUFB + dstb[u]) = rh[slot][u];
            *reinterpret_cast<u32x4_t*>(Bl + buf * BUFB + dstb[u]) = rl[slot][u];
        }
    };
    auto stage = [&](int slot) {
        lds_barrier();   // the previous stripe is fully consumed
        put(slot, 0);
        lds_barrier();
    };
    const int wn = wave % WN, wm = wave / WN;
    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // One stripe = 2 k-steps x 4 groups of 16 activation rows.  The weight fragments of both k-steps are read up
    // front; the hi / lo fragments of step t + 1 are requested before the eight MFMAs of step t are issued, so the
    // LDS latency hides behind the matrix pipe.  No conditions inside (row groups past M multiply clamped copies of
    // the last row; their results are never stored): one straight-line block for the scheduler.
    const unsigned char* wfrag = Ws + (wn * 64 + r16) * MB_PITCH + g * 16;
    const unsigned char* hfrag = Bh + (wm * 64 + r16) * MB_PITCH + g * 16;
    const unsigned char* lfrag = Bl + (wm * 64 + r16) * MB_PITCH + g * 16;
    auto multiply = [&](int buf) {
        constexpr int KS = MB_CK / 32, NSTEP = KS * 4;
        u32x4_t a[KS][4], h[2], l[2];
        const int bo = buf * BUFB;
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
#pragma unroll
            for (int i = 0; i < 4; i++) a[ks][i] = *reinterpret_cast<const u32x4_t*>(wfrag + bo + i * 16 * MB_PITCH + ks * 64);
        h[0] = *reinterpret_cast<const u32x4_t*>(hfrag + bo);
        l[0] = *reinterpret_cast<const u32x4_t*>(lfrag + bo);
#pragma unroll
        for (int t = 0; t < NSTEP; t++) {
            const int ks = t >> 2, j = t & 3;
            if (t + 1 < NSTEP) {
                const int o = bo + ((t + 1) & 3) * 16 * MB_PITCH + ((t + 1) >> 2) * 64;
                h[(t + 1) & 1] = *reinterpret_cast<const u32x4_t*>(hfrag + o);
                l[(t + 1) & 1] = *reinterpret_cast<const u32x4_t*>(lfrag + o);
            }
#pragma unroll
            for (int i = 0; i < 4; i++) acc[i][j] = mfma_h16<F16>(a[ks][i], h[t & 1], acc[i][j]);
#pragma unroll
            for (int i = 0; i < 4; i++) acc[i][j] = mfma_h16<F16>(a[ks][i], l[t & 1], acc[i][j]);
        }
    };
#pragma unroll
    for (int sl = 0; sl < MB_D; sl++)
        if (sl < NC) gload(sl, sl);
    // RMS scale of the block's activation rows from the producer's per-tile sums of squares (a K-split launch leaves
    // the scaling to its finishing kernel)
    if (tid < MB_TM) rs[tid] = 1.0f;
    if (MODE != RM_RESID && p.ssq && S == 1) {
        __syncthreads();
        for (int c = wave; c < MB_TM; c += NTH / 64) {
            const int m = min(m0 + c, M - 1);
            float sq = 0.f;
            for (int i = lane; i < p.n_ssq; i += 64) sq += p.ssq[(size_t)m * p.n_ssq + i];
            sq = wave_sum(sq);
            if (lane == 0) rs[c] = 1.0f / sqrtf(sq / (float)K + p.eps);
        }
    }
    if (NBUF == 1) {
        int ck0 = 0;
        for (; ck0 + 2 * MB_D <= NC; ck0 += MB_D) {   // steady state: every step refills its slot, no conditions
#pragma unroll
            for (int sl = 0; sl < MB_D; sl++) {
                stage(sl);
                gload(sl, ck0 + sl + MB_D);
                multiply(0);
            }
        }
        for (; ck0 < NC; ck0 += MB_D) {               // drain
#pragma unroll
            for (int sl = 0; sl < MB_D; sl++) {
                if (ck0 + sl < NC) {   // uniform
                    stage(sl);
                    if (ck0 + sl + MB_D < NC) gload(sl, ck0 + sl + MB_D);
                    multiply(0);
                }
            }
        }
    } else {
        // Two staging buffers: stripe c is multiplied out of buffer c % 2 while stripe c + 1 is written into the other
        // one and stripe c + 2 is on its way from memory; one barrier per stripe.  (Buffer (c + 1) % 2 was last read
        // for stripe c - 1, which every wave finished before the barrier that ended step c - 1.)
        if (NC > 0) put(0, 0);
        lds_barrier();
        int ck0 = 0;
        for (; ck0 + 2 * MB_D <= NC; ck0 += MB_D) {   // steady state, no conditions (MB_D = 2: slot = buffer = parity)
#pragma unroll
            for (int sl = 0; sl < MB_D; sl++) {
                gload(sl, ck0 + sl + MB_D);           // slot sl was stored to LDS one step ago
                multiply(sl);
                put(sl ^ 1, sl ^ 1);                  // stripe ck0 + sl + 1, requested two steps ago
                lds_barrier();
            }
        }
        for (; ck0 < NC; ck0 += MB_D) {               // drain
#pragma unroll
            for (int sl = 0; sl < MB_D; sl++) {
                if (ck0 + sl < NC) {   // uniform
                    if (ck0 + sl + MB_D < NC) gload(sl, ck0 + sl + MB_D);
                    multiply(sl);
                    if (ck0 + sl + 1 < NC) put(sl ^ 1, sl ^ 1);
                    lds_barrier();
                }
            }
        }
    }
    // epilogue, 64 activation rows at a time: ep[row][column] through LDS, then thread -> (column n, rows mm, mm + 2, ..)
    float* ep = reinterpret_cast<float*>(smb);
    const int n = tid % TN, mm = tid / TN;
    for (int hf = 0; hf < 2; hf++) {
        if (m0 + hf * 64 >= M) break;   // uniform over the block
        __syncthreads();
        if (wm == hf) {
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++)
                    *reinterpret_cast<f32x4_t*>(ep + (j * 16 + r16) * EP + wn * 64 + i * 16 + 4 * g) = acc[i][j];
        }
        __syncthreads();
        for (int it = 0; it < 32; it++) {
            const int ml = mm + 2 * it, m = m0 + hf * 64 + ml;   // uniform over a wave
            if (m >= M) break;
            float v = ep[ml * EP + n];
            if (S > 1) {   // raw sums of this K slice: [slice][matrix][M][columns of this launch's tiles]
                if (MODE == RM_SWIGLU)
                    p.kpart[(((size_t)slice * 2 + n / (TN / 2)) * M + m) * ((size_t)p.n_tiles * (TN / 2)) +
                            (size_t)(tile - p.tile0) * (TN / 2) + n % (TN / 2)] = v;
                else
                    p.kpart[((size_t)slice * M + m) * ((size_t)p.n_tiles * TN) + (size_t)(tile - p.tile0) * TN + n] = v;
                continue;
            }
            const float sc = rs[hf * 64 + ml];
            if (MODE == RM_STORE) {
                p.y[(size_t)m * p.ldy + (size_t)tile * TN + n] = v * sc;
            } else if (MODE == RM_SWIGLU) {
                if (n < TN / 2) {
                    const float gt = v * sc, up = ep[ml * EP + n + TN / 2] * sc;
                    split_store(gt / (1.0f + __expf(-gt)) * up, p.oh, p.ol, (size_t)m * p.ldo + (size_t)tile * (TN / 2) + n, F16);
                }
            } else if (MODE == RM_RESID) {
                const size_t colx = (size_t)tile * TN + n;
                float* dsty = p.y + (size_t)m * p.ldy + colx;
                const float tv = *dsty + v;
                *dsty = tv;
                if (p.tap && (p.tap_only <= 0 || m == p.tap_only - 1)) p.tap[(size_t)(p.tap_only > 0 ? 0 : m) * p.tap_ld + colx] = tv;
                if (p.gain_out) {
                    split_store(tv * p.gain_out[colx], p.oh, p.ol, (size_t)m * p.ldo + colx, F16);
                    const float sq = wave_sum(tv * tv);   // the wave holds 64 consecutive columns of row m
                    if (lane == 0) p.ssq_out[(size_t)m * (p.n[0] >> 6) + tile * WN + (n >> 6)] = sq;
                }
            } else {   // QKV: natural row order, the rotary partner of column n is n ^ (hd / 2) of the same tile
                const int row = tile * TN + n;
                const int pos = p.pos_dev[0] + p.pos_off + m;
                v *= sc;
                if (row < p.dq + p.dkv) {
                    const bool is_q = row < p.dq;
                    const int jj = is_q ? row : row - p.dq;
                    const int head = jj / p.hd, e = jj % p.hd, half = p.hd >> 1, i = e % half;
                    const float other = ep[ml * EP + (n ^ half)] * sc;
                    const float* cs = p.rope + ((size_t)pos * half + i) * 2;
                    const float ov = e < half ? v * cs[0] - other * cs[1] : v * cs[0] + other * cs[1];
                    if (is_q) p.y[(size_t)m * p.ldy + (size_t)head * p.hd + e] = ov;
                    else kv_put(p.kc, ((size_t)head * p.max_seq + pos) * p.hd + e, ov, p.kt);
                } else {
                    const int e = row - p.dq - p.dkv;
                    kv_put(p.vc, ((size_t)(e / p.hd) * p.max_seq + pos) * p.hd + (e % p.hd), v, p.kt);
                }
            }
        }
    }
}

// Second half of a K-split QKV launch of the large tiles (weight rows in natural order): one wave per (row, 64
// columns) adds the slices of its column and of the column's rotary partner in a fixed order, scales both by the row's
// RMS factor, rotates and writes the query row / the cache rows.
template <bool F16>
__global__ __launch_bounds__(64) void rows_finish_qkv_kernel(RowsP2 p)
{
    const int m = blockIdx.y, lane = threadIdx.x, half = p.hd >> 1;
    const size_t nt = (size_t)gridDim.x * 64;
    const int col = blockIdx.x * 64 + lane, row = p.fin_tile0 * 64 + col;
    const bool rotary = row < p.dq + p.dkv;   // uniform over the wave (dq, dkv are multiples of 128)
    float v = 0.f, other = 0.f;
    for (int sl = 0; sl < p.ksplit; sl++) {
        const float* src = p.kpart + ((size_t)sl * p.M + m) * nt;
        v += src[col];
        if (rotary) other += src[col ^ half];
    }
    if (p.ssq) {
        float sq = 0.f;
        for (int i = lane; i < p.n_ssq; i += 64) sq += p.ssq[(size_t)m * p.n_ssq + i];
        const float sc = 1.0f / sqrtf(wave_sum(sq) / (float)p.K + p.eps);
        v *= sc; other *= sc;
    }
    const int pos = p.pos_dev[0] + p.pos_off + m;
    if (rotary) {
        const bool is_q = row < p.dq;
        const int jj = is_q ? row : row - p.dq;
        const int head = jj / p.hd, e = jj % p.hd, i = e % half;
        const float* cs = p.rope + ((size_t)pos * half + i) * 2;
        const float ov = e < half ? v * cs[0] - other * cs[1] : v * cs[0] + other * cs[1];
        if (is_q) p.y[(size_t)m * p.ldy + (size_t)head * p.hd + e] = ov;
        else kv_put(p.kc, ((size_t)head * p.max_seq + pos) * p.hd + e, ov, p.kt);
    } else {
        const int e = row - p.dq - p.dkv;
        kv_put(p.vc, ((size_t)(e / p.hd) * p.max_seq + pos) * p.hd + (e % p.hd), v, p.kt);
    }
}

bool rows_big_supported(const Dims& D)
{
    return D.wt != WT_F32 && D.d % 128 == 0 && D.dq % 128 == 0 && D.dkv % 128 == 0 && D.f % 64 == 0 && D.V % 128 == 0 &&
           (D.hd == 64 || D.hd == 128);
}

bool rows_many_supported(const Dims& D, int N, int K)
{
    return D.wt != WT_F32 && N % 64 == 0 && K % M6_CK == 0 && K >= M6_CK;
}

// every GEMM of a layer and the LM head fit the 64 x 64 x 128 tiling
bool rows_wide_supported(const Dims& D)
{
    return D.wt != WT_F32 && D.d % 128 == 0 && D.dq % 128 == 0 && D.f % 128 == 0 && D.dkv % 64 == 0 && D.V % 64 == 0 &&
           (D.hd == 64 || D.hd == 128);
}

template <int MODE, bool F16, int DEPTH>
static hipError_t launch_wide_d(const RowsP2& p, int n_tiles, hipStream_t s)
{
    constexpr int NT = MODE == RM_SWIGLU ? 2 : 1;
    const size_t lds = (size_t)(NT * 64 + 128) * M6_PITCH;
    static std::atomic<size_t> lds_limit{0};  // per instantiation
    {
        hipError_t e = ensure_lds((const void*)rows_wide_kernel<MODE, F16, DEPTH>, lds, lds_limit);
        if (e != hipSuccess) return e;
    }
    const int S = p.ksplit > 1 ? p.ksplit : 1;
    hipLaunchKernelGGL((rows_wide_kernel<MODE, F16, DEPTH>), dim3(n_tiles, S), dim3(512), lds, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || S == 1) return e;
    hipLaunchKernelGGL((rows_finish_kernel<MODE, F16>), dim3(n_tiles, (p.M + FIN_ROWS - 1) / FIN_ROWS), dim3(64), 0, s, p);
    return hipGetLastError();
}

// One stripe in flight per block measured best or equal everywhere: what bounds a block is the 40 GB/s or so
// that a single CU pulls from the cache (a stripe is 48-64 KB of weights and rows), not latency.
template <int MODE, bool F16>
static hipError_t launch_wide(const RowsP2& p, int n_tiles, hipStream_t s, const LaunchOpts* opt)
{
    const int depth = opt && opt->wide_depth > 0 ? opt->wide_depth : 1;
    if (depth >= 4) return launch_wide_d<MODE, F16, 4>(p, n_tiles, s);
    if (depth >= 2) return launch_wide_d<MODE, F16, 2>(p, n_tiles, s);
    return launch_wide_d<MODE, F16, 1>(p, n_tiles, s);
}

static void fill_rows_params(const Dims& D, const RowsFused& f, RowsP2& p)
{
    for (int i = 0; i < 3; i++) { p.w[i] = f.w[i]; p.n[i] = f.n[i]; }
    p.K = f.K; p.bh = f.bh; p.bl = f.bl; p.ldb = f.ldb; p.y = f.y; p.ldy = f.ldy; p.oh = f.oh; p.ol = f.ol; p.ldo = f.ldo;
    p.tap = f.tap; p.tap_ld = f.tap_ld; p.M = f.M; p.rope = f.rope; p.pos_dev = f.pos_dev; p.pos_off = f.pos_off;
    p.hd = D.hd; p.dq = D.dq; p.dkv = D.dkv; p.max_seq = D.max_seq; p.kc = f.kc; p.vc = f.vc; p.kt = D.kt;
    p.ssq = f.ssq; p.n_ssq = f.n_ssq; p.eps = D.eps; p.gain_out = f.gain_out; p.ssq_out = f.ssq_out;
    p.tap_only = f.tap_only;
}

hipError_t rows_wide(const Dims& D, const RowsFused& f, hipStream_t s)
{
    if (D.wt == WT_F32 || f.M < 1 || f.M > 64 || f.K % M6_CK || f.K < M6_CK) return hipErrorInvalidValue;
    if (f.n[0] % 64 || f.n[1] % 64 || f.n[2] % 64) return hipErrorInvalidValue;
    if (f.ssq && (f.mode == RM_RESID || f.n_ssq < 1)) return hipErrorInvalidValue;
    if (f.gain_out && (f.mode != RM_RESID || !f.oh || !f.ol || !f.ssq_out)) return hipErrorInvalidValue;
    if (f.mode == RM_QKV && (f.n[0] != D.dq || f.n[1] != D.dkv || f.n[2] != D.dkv || (D.hd != 64 && D.hd != 128)))
        return hipErrorInvalidValue;
    RowsP2 p = {};
    fill_rows_params(D, f, p);
    const int n_tiles = f.mode == RM_SWIGLU ? f.n[0] / 64 : (f.n[0] + f.n[1] + f.n[2]) / 64;
    const bool f16 = D.wt == WT_F16;
    // A block is bound by what one CU pulls from the cache (about 40 GB/s), so a launch with far fewer tiles than
    // CUs (the projections back to d_model) is cut along K until there are about 256 blocks; needs scratch for
    // ksplit x matrices x M x n sums.  With 170 tiles or more (QKV, gate/up at 7B) the cut measured equal or worse.
    p.ksplit = 1; p.kpart = nullptr;
    const int force_ks = D.opt ? D.opt->wide_ksplit : 0;
    if (f.kpart && force_ks != 1 && f.M > 16) {
        const int nmat = f.mode == RM_SWIGLU ? 2 : 1;
        const size_t per_slice = (size_t)nmat * f.M * n_tiles * 64;
        int ks = force_ks > 1 ? force_ks : (n_tiles <= 128 ? 256 / n_tiles : 1);
        const int nc = f.K / M6_CK;
        if (ks > 8) ks = 8;
        if (ks > nc) ks = nc;
        if ((size_t)ks * per_slice > f.kpart_floats) ks = (int)(f.kpart_floats / per_slice);
        if (ks > 1) { p.ksplit = ks; p.kpart = f.kpart; }
    }
    switch (f.mode) {
        case RM_STORE: return f16 ? launch_wide<RM_STORE, true>(p, n_tiles, s, D.opt) : launch_wide<RM_STORE, false>(p, n_tiles, s, D.opt);
        case RM_RESID: return f16 ? launch_wide<RM_RESID, true>(p, n_tiles, s, D.opt) : launch_wide<RM_RESID, false>(p, n_tiles, s, D.opt);
        case RM_SWIGLU: return f16 ? launch_wide<RM_SWIGLU, true>(p, n_tiles, s, D.opt) : launch_wide<RM_SWIGLU, false>(p, n_tiles, s, D.opt);
        case RM_QKV: return f16 ? launch_wide<RM_QKV, true>(p, n_tiles, s, D.opt) : launch_wide<RM_QKV, false>(p, n_tiles, s, D.opt);
        default: return hipErrorInvalidValue;
    }
}

template <int MODE, bool F16, int TN>
static hipError_t launch_big(const RowsP2& p, hipStream_t s)
{
    const size_t lds = (size_t)(TN == 256 ? 2 : 1) * (TN + 2 * MB_TM) * MB_PITCH;
    static_assert((size_t)64 * (TN + 4) * 4 <= (size_t)(TN + 2 * MB_TM) * MB_PITCH, "epilogue tile fits the staging area");
    static std::atomic<size_t> lds_limit{0};  // per instantiation
    {
        hipError_t e = ensure_lds((const void*)rows_big_kernel<MODE, F16, TN>, lds, lds_limit);
        if (e != hipSuccess) return e;
    }
    const int S = p.ksplit > 1 ? p.ksplit : 1;
    hipLaunchKernelGGL((rows_big_kernel<MODE, F16, TN>), dim3(p.n_tiles * ((p.M + MB_TM - 1) / MB_TM) * S), dim3(TN * 2), lds, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || S == 1) return e;
    if (MODE == RM_QKV)   // natural row order: its own finishing kernel
        hipLaunchKernelGGL((rows_finish_qkv_kernel<F16>), dim3(p.n_tiles * (TN / 64), p.M), dim3(64), 0, s, p);
    else
        hipLaunchKernelGGL((rows_finish_kernel<MODE, F16>), dim3(p.n_tiles * (MODE == RM_SWIGLU ? TN / 128 : TN / 64), (p.M + FIN_ROWS - 1) / FIN_ROWS), dim3(64), 0, s, p);
    return hipGetLastError();
}

template <int MODE, bool F16>
static hipError_t launch_big_tn(const RowsP2& p, int tn, hipStream_t s)
{
    return tn == 256 ? launch_big<MODE, F16, 256>(p, s) : launch_big<MODE, F16, 128>(p, s);
}

hipError_t rows_big(const Dims& D, const RowsFused& f, hipStream_t s)
{
    if (D.wt == WT_F32 || f.M < 1 || f.K % MB_CK || f.K < MB_CK) return hipErrorInvalidValue;
    if (f.mode == RM_SWIGLU ? (f.n[0] % 64 || f.n[1] != f.n[0]) : (f.n[0] % 128 || f.n[1] % 128 || f.n[2] % 128))
        return hipErrorInvalidValue;
    if (f.ssq && (f.mode == RM_RESID || f.n_ssq < 1)) return hipErrorInvalidValue;
    if (f.gain_out && (f.mode != RM_RESID || !f.oh || !f.ol || !f.ssq_out)) return hipErrorInvalidValue;
    if (f.mode == RM_QKV && (f.n[0] != D.dq || f.n[1] != D.dkv || f.n[2] != D.dkv || (D.hd != 64 && D.hd != 128)))
        return hipErrorInvalidValue;
    RowsP2 p = {};
    fill_rows_params(D, f, p);
    const int m_blocks = (f.M + MB_TM - 1) / MB_TM;
    const int n_total = f.mode == RM_SWIGLU ? 2 * f.n[0] : f.n[0] + f.n[1] + f.n[2];   // logical weight rows
    // 256-row tiles (one 512-thread block per CU, staging double-buffered in LDS: measured 20-30 % faster per MFMA, and
    // a launch fills the CUs with the same granularity as two 128-row blocks per CU would) wherever every stacked
    // matrix is a whole number of them; else 128-row tiles
    const int force_tn = D.opt ? D.opt->wide_depth : 0;   // tuning hook: 128 or 256
    const bool fits256 = f.mode == RM_SWIGLU ? f.n[0] % 128 == 0 : (f.n[0] % 256 == 0 && f.n[1] % 256 == 0 && f.n[2] % 256 == 0);
    int tn = fits256 ? 256 : 128;
    if (force_tn == 128 || (force_tn == 256 && fits256)) tn = force_tn;
    const int n_tiles = n_total / tn;
    p.n_tiles = n_tiles;
    const bool f16 = D.wt == WT_F16;
    // a residual projection with fewer blocks than resident slots (two per CU for the small tile, one for the large)
    // is cut along K (its raw sums go to kpart and rows_finish_kernel adds the slices in a fixed order)
    p.ksplit = 1; p.kpart = nullptr;
    const int force_ks = D.opt ? D.opt->wide_ksplit : 0;
    if (f.kpart && f.mode == RM_RESID && force_ks != 1) {
        const size_t per_slice = (size_t)f.M * n_tiles * tn;
        int ks = force_ks > 1 ? force_ks : (tn == 256 ? 256 : 512) / (n_tiles * m_blocks);
        const int nc = f.K / MB_CK;
        if (ks > 8) ks = 8;
        if (ks > nc) ks = nc;
        if ((size_t)ks * per_slice > f.kpart_floats) ks = (int)(f.kpart_floats / per_slice);
        if (ks > 1) { p.ksplit = ks; p.kpart = f.kpart; }
    }
    // A QKV launch with blocks for at most half of the slots (prompts of up to 256 rows at the 7B shape) is cut along K
    // as well; its finishing kernel rotates and writes the cache rows.
    if (f.kpart && f.mode == RM_QKV && force_ks != 1) {
        const int slots = tn == 256 ? 256 : 512, nc = f.K / MB_CK;
        const size_t per_slice = (size_t)f.M * n_tiles * tn;
        int ks = force_ks > 1 ? force_ks : slots / (n_tiles * m_blocks);
        if (ks > 4) ks = 4;
        if (ks > nc) ks = nc;
        if ((size_t)ks * per_slice > f.kpart_floats) ks = (int)(f.kpart_floats / per_slice);
        if (ks > 1) { p.ksplit = ks; p.kpart = f.kpart; }
    }
    // Gate / up with a last round that would leave most CUs idle (7B, 512 rows: 344 blocks for 256 slots): the tiles
    // of the whole rounds run as they are, the rest (all of them when there is no whole round) are cut along K into as
    // many slices as fill the slots once more, and the finishing kernel adds the slices and applies SwiGLU
    // (1 + 1/2 block times instead of 2).
    if (f.kpart && f.mode == RM_SWIGLU && force_ks != 1) {
        const int slots = tn == 256 ? 256 : 512, units = n_tiles * m_blocks;
        const int whole_tiles = units / slots * slots / m_blocks, tail_tiles = n_tiles - whole_tiles;
        const int tail_units = tail_tiles * m_blocks, nc = f.K / MB_CK;
        if (tail_tiles > 0) {
            int ks = slots / tail_units;
            if (ks > 4) ks = 4;
            if (ks > nc) ks = nc;
            const size_t per_slice = (size_t)2 * f.M * tail_tiles * (tn / 2);
            if ((size_t)ks * per_slice > f.kpart_floats) ks = (int)(f.kpart_floats / per_slice);
            if (ks > 1) {
                if (whole_tiles > 0) {
                    RowsP2 a = p;
                    a.n_tiles = whole_tiles;
                    const hipError_t e = f16 ? launch_big_tn<RM_SWIGLU, true>(a, tn, s) : launch_big_tn<RM_SWIGLU, false>(a, tn, s);
                    if (e != hipSuccess) return e;
                }
                p.tile0 = whole_tiles; p.n_tiles = tail_tiles; p.fin_tile0 = whole_tiles * (tn / 128);
                p.ksplit = ks; p.kpart = f.kpart;
            }
        }
    }
    switch (f.mode) {
        case RM_STORE: return f16 ? launch_big_tn<RM_STORE, true>(p, tn, s) : launch_big_tn<RM_STORE, false>(p, tn, s);
        case RM_RESID: return f16 ? launch_big_tn<RM_RESID, true>(p, tn, s) : launch_big_tn<RM_RESID, false>(p, tn, s);
        case RM_SWIGLU: return f16 ? launch_big_tn<RM_SWIGLU, true>(p, tn, s) : launch_big_tn<RM_SWIGLU, false>(p, tn, s);
        case RM_QKV: return f16 ? launch_big_tn<RM_QKV, true>(p, tn, s) : launch_big_tn<RM_QKV, false>(p, tn, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t rows_many(const Dims& D, const void* w, int N, int K, const uint16_t* bh, const uint16_t* bl, int ldb, int M,
                     float* y, int ldy, hipStream_t s)
{
    if (!rows_many_supported(D, N, K)) return hipErrorInvalidValue;
    RowsFused f = {};
    f.w[0] = w; f.n[0] = N; f.K = K; f.bh = bh; f.bl = bl; f.ldb = ldb; f.y = y; f.ldy = ldy; f.M = M; f.mode = RM_STORE;
    return rows_wide(D, f, s);
}

bool rows_fused_supported(const Dims& D)
{
    return D.wt != WT_F32 && D.d % 64 == 0 && D.dq % 64 == 0 && D.f % 64 == 0;
}

hipError_t rows_fused(const Dims& D, const RowsFused& f, hipStream_t s)
{
    if (!rows_fused_supported(D) || f.M < 1 || f.M > 16 || f.K % 64) return hipErrorInvalidValue;
    RowsP2 p = {};
    fill_rows_params(D, f, p);
    if (f.ssq && (f.mode == RM_RESID || f.n_ssq < 1)) return hipErrorInvalidValue;
    if (f.gain_out && (f.mode != RM_RESID || !f.oh || !f.ol || !f.ssq_out)) return hipErrorInvalidValue;
    switch (f.mode) {
        case RM_STORE: return D.wt == WT_F16 ? rows_fused_mode<RM_STORE, true>(p, s, D.opt) : rows_fused_mode<RM_STORE, false>(p, s, D.opt);
        case RM_RESID: return D.wt == WT_F16 ? rows_fused_mode<RM_RESID, true>(p, s, D.opt) : rows_fused_mode<RM_RESID, false>(p, s, D.opt);
        case RM_SWIGLU: return D.wt == WT_F16 ? rows_fused_mode<RM_SWIGLU, true>(p, s, D.opt) : rows_fused_mode<RM_SWIGLU, false>(p, s, D.opt);
        case RM_QKV: return D.wt == WT_F16 ? rows_fused_mode<RM_QKV, true>(p, s, D.opt) : rows_fused_mode<RM_QKV, false>(p, s, D.opt);
    }
    return hipErrorInvalidValue;
}

// hi/lo bf16 split of M rows of length K, optionally RMS-normalised first (gain != nullptr)
__global__ __launch_bounds__(256) void rows_prep_kernel(const float* __restrict__ in, int ldx, const float* __restrict__ gain,
                                                        int K, float eps, uint16_t* __restrict__ hi, uint16_t* __restrict__ lo,
                                                        bool f16)
{
    __shared__ float red[4];
    const float* x = in + (size_t)blockIdx.x * ldx;
    float sc = 1.0f;
    if (gain) {
        float ss = 0.f;
        for (int i = threadIdx.x * 4; i < K; i += 1024) {
            const float4 v = *reinterpret_cast<const float4*>(x + i);
            ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        }
        sc = 1.0f / sqrtf(block_sum<4>(ss, red) / (float)K + eps);
    }
    for (int i = threadIdx.x * 4; i < K; i += 1024) {
        float4 v = *reinterpret_cast<const float4*>(x + i);
        if (gain) {
            const float4 g = *reinterpret_cast<const float4*>(gain + i);
            v.x = v.x * sc * g.x; v.y = v.y * sc * g.y; v.z = v.z * sc * g.z; v.w = v.w * sc * g.w;
        }
        const size_t o = (size_t)blockIdx.x * K + i;
        split_store(v.x, hi, lo, o, f16); split_store(v.y, hi, lo, o + 1, f16);
        split_store(v.z, hi, lo, o + 2, f16); split_store(v.w, hi, lo, o + 3, f16);
    }
}

hipError_t rows_prep(const Dims& D, const float* in, int ldx, const float* gain, int M, int K, float eps, uint16_t* hi,
                     uint16_t* lo, hipStream_t s)
{
    hipLaunchKernelGGL(rows_prep_kernel, dim3(M), dim3(256), 0, s, in, ldx, gain, K, eps, hi, lo, D.wt == WT_F16);
    return hipGetLastError();
}

// Entry of the fused path (rows straight from the embedding): hi/lo = split(x * gain) without the
// norm scale, and the sums of squares of every `group` (16 or 64) consecutive elements, i.e. exactly what a
// RESID projection with tiles of that width leaves behind for its consumer.
__global__ __launch_bounds__(256) void rows_gain_split_kernel(const float* __restrict__ in, int ldx,
                                                              const float* __restrict__ gain, int K,
                                                              uint16_t* __restrict__ hi, uint16_t* __restrict__ lo,
                                                              float* __restrict__ ssq, bool f16, int group)
{
    const float* x = in + (size_t)blockIdx.x * ldx;
    const int n_t = K / group;
    for (int t = threadIdx.x; t < n_t; t += 256) {
        float sq = 0.f;
        for (int u = 0; u < group; u += 4) {
            const int i = t * group + u;
            const float4 v = *reinterpret_cast<const float4*>(x + i);
            const float4 g = *reinterpret_cast<const float4*>(gain + i);
            sq += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            const size_t o = (size_t)blockIdx.x * K + i;
            split_store(v.x * g.x, hi, lo, o, f16); split_store(v.y * g.y, hi, lo, o + 1, f16);
            split_store(v.z * g.z, hi, lo, o + 2, f16); split_store(v.w * g.w, hi, lo, o + 3, f16);
        }
        ssq[(size_t)blockIdx.x * n_t + t] = sq;
    }
}

hipError_t rows_gain_split(const Dims& D, const float* in, int ldx, const float* gain, int M, int K, uint16_t* hi, uint16_t* lo,
                           float* ssq, int group, hipStream_t s)
{
    if ((group != 16 && group != 64) || K % group || !gain) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rows_gain_split_kernel, dim3(M), dim3(256), 0, s, in, ldx, gain, K, hi, lo, ssq, D.wt == WT_F16, group);
    return hipGetLastError();
}

// rotary + cache write for the multi-row path: one thread per (row, head slot, pair index)
template <typename KT>
__global__ void rope_kv_rows_kernel(float* __restrict__ qkv, const float* __restrict__ rope, const int* pos_dev,
                                    int pos_off, int M, int H, int Hkv, int hd, int max_seq, KT* __restrict__ kc,
                                    KT* __restrict__ vc)
{
    const int half = hd >> 1;
    const int dq = H * hd, dkv = Hkv * hd, ld = dq + 2 * dkv;
    const int per_row = (H + Hkv) * half + dkv;  // q pairs, k pairs, v elements
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= M * per_row) return;
    int r = idx / per_row, e = idx % per_row;
    int pos = pos_dev[0] + pos_off + r;
    float* row = qkv + (size_t)r * ld;
    if (e < (H + Hkv) * half) {
        int hs = e / half, i = e % half;  // head slot over q heads then k heads
        const float* cs = rope + ((size_t)pos * half + i) * 2;
        float c = cs[0], s = cs[1];
        if (hs < H) {
            float* v = row + (size_t)hs * hd;
            float a = v[i], b = v[i + half];
            v[i] = a * c - b * s;
            v[i + half] = b * c + a * s;
        } else {
            int kvh = hs - H;
            const float* v = row + dq + (size_t)kvh * hd;
            float a = v[i], b = v[i + half];
            size_t o = ((size_t)kvh * max_seq + pos) * hd;
            Elem<KT>::put(kc, o + i, a * c - b * s);
            Elem<KT>::put(kc, o + i + half, b * c + a * s);
        }
    } else {
        int j = e - (H + Hkv) * half;  // element of v
        int kvh = j / hd, i = j % hd;
        Elem<KT>::put(vc, ((size_t)kvh * max_seq + pos) * hd + i, row[dq + dkv + j]);
    }
}

hipError_t rope_kv_rows(const Dims& D, float* qkv, const float* rope, const int* pos_dev, int pos_off, int M, void* kc,
                        void* vc, hipStream_t s)
{
    int per_row = (D.H + D.Hkv) * (D.hd / 2) + D.dkv;
    int blocks = ceil_div(M * per_row, 256);
    if (D.kt == WT_BF16)
        hipLaunchKernelGGL(rope_kv_rows_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, qkv, rope, pos_dev, pos_off, M,
                           D.H, D.Hkv, D.hd, D.max_seq, (uint16_t*)kc, (uint16_t*)vc);
    else if (D.kt == WT_F16)
        hipLaunchKernelGGL(rope_kv_rows_kernel<f16_t>, dim3(blocks), dim3(256), 0, s, qkv, rope, pos_dev, pos_off, M,
                           D.H, D.Hkv, D.hd, D.max_seq, (f16_t*)kc, (f16_t*)vc);
    else
        hipLaunchKernelGGL(rope_kv_rows_kernel<float>, dim3(blocks), dim3(256), 0, s, qkv, rope, pos_dev, pos_off, M, D.H,
                           D.Hkv, D.hd, D.max_seq, (float*)kc, (float*)vc);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// attention over the cache: split over the sequence, K/V tiles staged through LDS
// ---------------------------------------------------------------------------------------------
constexpr int AT_THREADS = 256;
constexpr int AT_CHUNK = 96;   // cache positions one block owns (K and V of the chunk live in LDS together)
constexpr int AT_QPASS = 16;   // query vectors handled per pass over the staged chunk

// P.V for up to NQ query vectors at once: acc[qi] += e[qi][j] * V[j][d] over this thread's positions
template <typename KT, int NQ>
__device__ __forceinline__ void attn_pv(const KT* vtile, int rowb, const float* sc, int d, int grp, int ng, int n,
                                        float (&acc)[AT_QPASS])
{
    for (int j = grp; j < n; j += ng) {
        const float v = Elem<KT>::get(reinterpret_cast<const KT*>(reinterpret_cast<const unsigned char*>(vtile) + (size_t)j * rowb), d);
#pragma unroll
        for (int qi = 0; qi < NQ; qi++) acc[qi] = fmaf(sc[qi * AT_CHUNK + j], v, acc[qi]);
    }
}

// One block = one KV head x one chunk of positions x ALL query vectors that read this head (the G
// query heads of the group times the M rows), so K and V are fetched once however many rows verify.
// All global loads of the chunk are issued up front, land in LDS (rows padded by 16 bytes to spread
// banks), and the three phases -- scores, softmax statistics, P.V -- then run out of LDS only.
// partial layout per (row, head, split): [hd] unnormalised output, then m (max score), l (sum of exp), 2 pad
// (stride hd + 4 floats keeps every partial 16-byte aligned)
template <typename KT, int HD>
__global__ __launch_bounds__(AT_THREADS) void attn_kernel(const float* __restrict__ q, int ldq,
                                                          const KT* __restrict__ kc, const KT* __restrict__ vc,
                                                          const int* pos_dev, int pos_off, int M, int H, int Hkv,
                                                          int max_seq, int n_splits, float* __restrict__ part,
                                                          float* __restrict__ outp, int dq,
                                                          uint16_t* __restrict__ out_hi, uint16_t* __restrict__ out_lo,
                                                          bool out_f16)
{
    constexpr int ROWB = HD * (int)sizeof(KT) + 16;
    constexpr int EPV = 16 / (int)sizeof(KT);  // elements per 16-byte vector
    constexpr int VPR = HD / EPV;              // vectors per cache row
    constexpr int NG = AT_THREADS / HD;        // position groups in the P.V phase
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* ktile = smem;
    unsigned char* vtile = smem + AT_CHUNK * ROWB;
    float* qs = reinterpret_cast<float*>(smem + 2 * AT_CHUNK * ROWB);  // [AT_QPASS][HD], pre-scaled
    float* sc = qs + AT_QPASS * HD;                                    // [AT_QPASS][AT_CHUNK]
    float* ml = sc + AT_QPASS * AT_CHUNK;                              // [AT_QPASS][2]
    float* fold = ml + AT_QPASS * 2;                                   // [NG][AT_QPASS][HD]

    const int split = blockIdx.x, kvh = blockIdx.y;
    const int G = H / Hkv, Q = G * M;
    const int p0 = pos_dev[0] + pos_off;
    const int total = p0 + M;                                  // positions the last row sees
    const int chunk = min((total + n_splits - 1) / n_splits, AT_CHUNK);  // host sizes n_splits so this is <= AT_CHUNK
    const int j0 = split * chunk;
    const int n = min(chunk, total - j0);                      // may be <= 0
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    if (n > 0) {  // stage K and V of the chunk: every load is issued before the first is used
        const KT* kbase = kc + ((size_t)kvh * max_seq + j0) * HD;
        const KT* vbase = vc + ((size_t)kvh * max_seq + j0) * HD;
        constexpr int NV = (AT_CHUNK * VPR + AT_THREADS - 1) / AT_THREADS;
        uint4 kr[NV], vr[NV];
        const int vmax = n * VPR - 1;
#pragma unroll
        for (int t = 0; t < NV; t++) {  // clamped, not predicated: the loads stay in registers and in flight together
            const int v = min(tid + t * AT_THREADS, vmax);
            kr[t] = *reinterpret_cast<const uint4*>(kbase + (size_t)(v / VPR) * HD + (v % VPR) * EPV);
            vr[t] = *reinterpret_cast<const uint4*>(vbase + (size_t)(v / VPR) * HD + (v % VPR) * EPV);
        }
#pragma unroll
        for (int t = 0; t < NV; t++) {
            const int v = tid + t * AT_THREADS;
            if (v <= vmax) {
                *reinterpret_cast<uint4*>(ktile + (v / VPR) * ROWB + (v % VPR) * 16) = kr[t];
                *reinterpret_cast<uint4*>(vtile + (v / VPR) * ROWB + (v % VPR) * 16) = vr[t];
            }
        }
    }
    const float scale = 1.0f / sqrtf((float)HD);
    for (int q0 = 0; q0 < Q; q0 += AT_QPASS) {   // uniform over the block
        const int nq = min(AT_QPASS, Q - q0);
        __syncthreads();                         // staged tiles visible / previous pass done with qs, sc
        for (int e = tid; e < nq * HD; e += AT_THREADS) {
            const int qi = q0 + e / HD, r = qi / G, g = qi % G;
            qs[e] = q[(size_t)r * ldq + (size_t)(kvh * G + g) * HD + (e % HD)] * scale;
        }
        __syncthreads();
        if (n > 0) {
            // phase A: scores. 2 lanes per position, each holding half a key row in registers
            constexpr int DPT = HD / 2;
            for (int jb = 0; jb < n; jb += AT_THREADS / 2) {
                const int j = jb + (tid >> 1), half = tid & 1;
                float kf[DPT];
                if (j < n) {
                    const KT* krow = reinterpret_cast<const KT*>(ktile + j * ROWB) + half * DPT;
#pragma unroll
                    for (int i = 0; i < DPT; i += EPV) {
                        float t8[EPV];
                        Elem<KT>::load(krow + i, t8);
#pragma unroll
                        for (int u = 0; u < EPV; u++) kf[i + u] = t8[u];
                    }
                }
                for (int qi = 0; qi < nq; qi++) {
                    float dot = 0.f;
                    if (j < n) {
                        const float* qv = qs + qi * HD + half * DPT;
#pragma unroll
                        for (int i = 0; i < DPT; i += 4) {
                            const float4 t4 = *reinterpret_cast<const float4*>(qv + i);
                            dot = fmaf(kf[i], t4.x, dot); dot = fmaf(kf[i + 1], t4.y, dot);
                            dot = fmaf(kf[i + 2], t4.z, dot); dot = fmaf(kf[i + 3], t4.w, dot);
                        }
                    }
                    dot += __shfl_xor(dot, 1, 64);
                    if (j < n && half == 0) sc[qi * AT_CHUNK + j] = dot;
                }
            }
        }
        __syncthreads();
        // phase B: per query vector (one wave each): causal mask, max, exp, sum
        for (int qi = wave; qi < nq; qi += AT_THREADS / 64) {
            const int r = (q0 + qi) / G;
            const int vis = min(n, p0 + r + 1 - j0);   // positions of this chunk the row may see
            float mx = -INFINITY;
            for (int j = lane; j < vis; j += 64) mx = fmaxf(mx, sc[qi * AT_CHUNK + j]);
            mx = wave_max(mx);
            float ls = 0.f;
            for (int j = lane; j < n; j += 64) {
                const float e = j < vis ? __expf(sc[qi * AT_CHUNK + j] - mx) : 0.f;
                sc[qi * AT_CHUNK + j] = e;
                ls += e;
            }
            ls = wave_sum(ls);
            if (lane == 0) { ml[qi * 2] = mx; ml[qi * 2 + 1] = ls; }
        }
        __syncthreads();
        // phase C: o[qi][d] = sum_j e[qi][j] V[j][d]; thread = (position group, d), all nq accumulators in registers
        const int d = tid % HD, grp = tid / HD;
        float acc[AT_QPASS];
#pragma unroll
        for (int qi = 0; qi < AT_QPASS; qi++) acc[qi] = 0.f;
        const KT* vcol = reinterpret_cast<const KT*>(vtile);
        if (nq == 1) attn_pv<KT, 1>(vcol, ROWB, sc, d, grp, NG, n, acc);
        else if (nq <= 4) attn_pv<KT, 4>(vcol, ROWB, sc, d, grp, NG, n, acc);
        else if (nq <= 8) attn_pv<KT, 8>(vcol, ROWB, sc, d, grp, NG, n, acc);
        else attn_pv<KT, AT_QPASS>(vcol, ROWB, sc, d, grp, NG, n, acc);
        // fold the NG position groups and write this split's result
#pragma unroll
        for (int qi = 0; qi < AT_QPASS; qi++)
            if (qi < nq) fold[(grp * AT_QPASS + qi) * HD + d] = acc[qi];
        __syncthreads();
        for (int e = tid; e < nq * HD; e += AT_THREADS) {
            const int qi = e / HD, dd = e % HD;
            float o = 0.f;
#pragma unroll
            for (int gg = 0; gg < NG; gg++) o += fold[(gg * AT_QPASS + qi) * HD + dd];
            const int qg = q0 + qi, r = qg / G, head = kvh * G + qg % G;
            const float mx = ml[qi * 2], ls = ml[qi * 2 + 1];
            if (n_splits == 1) {
                const size_t oo = (size_t)r * dq + (size_t)head * HD + dd;
                if (out_hi) split_store(o / ls, out_hi, out_lo, oo, out_f16);
                else outp[oo] = o / ls;
            } else {
                float* mine = part + (((size_t)r * H + head) * n_splits + split) * (HD + 4);
                mine[dd] = o;
                if (dd == 0) { mine[HD] = n > 0 ? mx : -INFINITY; mine[HD + 1] = ls; }
            }
        }
    }
}

// MFMA form of the kernel above for 16-bit caches: one block per KV head, chunk of positions and group of 16
// query vectors; same staging of K, same softmax statistics and the same partial layout, but the two
// contractions run on the matrix cores.  Scores: A = 16 query vectors (fp32 -> hi + lo in the cache's 16-bit
// type), B = K rows read from LDS in fragment order.  P.V: A = the 16 x 96 exponentials (hi + lo), B = V, which
// is therefore staged transposed ([dim][position]) so that a fragment is one 128-bit LDS read.
constexpr int AM_VPITCH = AT_CHUNK * 2 + 16;   // bytes per row of the transposed V tile

// 8 consecutive fp32 values -> two packed fragments hi = rne(x), lo = rne(x - hi)
template <bool F16>
__device__ __forceinline__ void split8(const float* x, u32x4_t& hi, u32x4_t& lo)
{
    // two 128-bit reads (x is 32-byte aligned), not eight dependent scalar ones
    const float4 a = *reinterpret_cast<const float4*>(x), b = *reinterpret_cast<const float4*>(x + 4);
    const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    unsigned h[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const uint16_t hb = f32_to_h16_bits(v[i], F16);
        h[i] = hb;
        l[i] = f32_to_h16_bits(v[i] - h16_bits_to_f32(hb, F16), F16);
    }
    hi = u32x4_t{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    lo = u32x4_t{l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
}

// fp32 caches take the same kernel: while a chunk is staged every K / V element is split into two bf16 planes
// (hi = rne(x), lo = rne(x - hi), 16 mantissa bits together), and each contraction becomes three MFMAs
// (hi.hi + lo.hi + hi.lo; the lo.lo term is below the 16 bits the planes carry).
template <typename KT, int HD>
__global__ __launch_bounds__(AT_THREADS) void attn_mfma_kernel(const float* __restrict__ q, int ldq,
                                                               const KT* __restrict__ kc, const KT* __restrict__ vc,
                                                               const int* pos_dev, int pos_off, int M, int H, int Hkv,
                                                               int max_seq, int n_splits, float* __restrict__ part,
                                                               float* __restrict__ outp, int dq,
                                                               uint16_t* __restrict__ out_hi, uint16_t* __restrict__ out_lo,
                                                               bool out_f16)
{
    constexpr bool F32 = sizeof(KT) == 4;
    constexpr bool F16 = IsF16<KT>::value;     // operand type of the MFMAs: fp16 for fp16 caches, else bf16
    constexpr int NP = F32 ? 2 : 1;            // planes per staged tile
    constexpr int ROWB = HD * 2 + 16;
    constexpr int EPV = 16 / (int)sizeof(KT);  // cache elements per 16-byte vector
    constexpr int VPR = HD / EPV;              // 16-byte vectors per cache row
    constexpr int KSTEPS = HD / 32;            // MFMA k-steps of a score
    constexpr int PT = AT_CHUNK / 16;          // position tiles of the chunk (6)
    constexpr int PS = AT_CHUNK / 32;          // k-steps of P.V (3)
    constexpr int DT = HD / 16;                // output dim tiles (8 or 4)
    constexpr int DTW = DT / 4;                // dim tiles per wave
    constexpr int KPLANE = AT_CHUNK * ROWB, VPLANE = HD * AM_VPITCH;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* ktile = smem;                                       // [NP][AT_CHUNK][ROWB]
    unsigned char* vT = smem + NP * KPLANE;                            // [NP][HD][AM_VPITCH]
    float* qs = reinterpret_cast<float*>(vT + NP * VPLANE);            // [16][HD], pre-scaled
    float* sc = qs + AT_QPASS * HD;                                    // [16][AT_CHUNK]
    float* ml = sc + AT_QPASS * AT_CHUNK;                              // [16][2]

    const int split = blockIdx.x, kvh = blockIdx.y;
    const int G = H / Hkv, Q = G * M;
    const int p0 = pos_dev[0] + pos_off;
    const int total = p0 + M;
    const int chunk = min((total + n_splits - 1) / n_splits, AT_CHUNK);
    const int j0 = split * chunk;
    const int n = min(chunk, total - j0);                      // may be <= 0
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    // the block's group of 16 query vectors (blockIdx.z): loads issued first, they are the furthest away
    const int q0 = blockIdx.z * AT_QPASS;
    const int nq = min(AT_QPASS, Q - q0);
    // A chunk that lies wholly behind the causal horizon of the block's LAST query row contributes nothing (in a
    // prompt pass that is half of all blocks): leave empty partials and go.  Uniform over the block.
    if (n_splits > 1 && (n <= 0 || j0 > p0 + (q0 + nq - 1) / G)) {
        for (int f = tid; f < nq * (HD / 4); f += AT_THREADS) {
            const int qi = f / (HD / 4), dd = (f % (HD / 4)) * 4;
            const int qg = q0 + qi, r = qg / G, head = kvh * G + qg % G;
            float* mine = part + (((size_t)r * H + head) * n_splits + split) * (HD + 4);
            *reinterpret_cast<float4*>(mine + dd) = make_float4(0.f, 0.f, 0.f, 0.f);
            if (dd == 0) { mine[HD] = -INFINITY; mine[HD + 1] = 0.f; }
        }
        return;
    }
    constexpr int QPT = AT_QPASS * HD / AT_THREADS;   // query elements per thread
    float qreg[QPT];
#pragma unroll
    for (int t = 0; t < QPT; t++) {
        const int e = tid + t * AT_THREADS, qg = q0 + min(e / HD, nq - 1);
        qreg[t] = q[(size_t)(qg / G) * ldq + (size_t)(kvh * G + qg % G) * HD + (e % HD)];
    }
    if (n > 0) {  // stage K (row-major) and V (transposed); every load is issued before the first is used
        const KT* kbase = kc + ((size_t)kvh * max_seq + j0) * HD;
        const KT* vbase = vc + ((size_t)kvh * max_seq + j0) * HD;
        constexpr int NV = (AT_CHUNK * VPR + AT_THREADS - 1) / AT_THREADS;
        u32x4_t kr[NV], vr[NV];
        const int vmax = n * VPR - 1;
        // K: consecutive lanes take consecutive vectors of a row.  V: consecutive lanes take consecutive POSITIONS
        // (vector v -> position v % AT_CHUNK, dims EPV (v / AT_CHUNK) ..), so that the 2-byte stores of the transpose
        // below fall on consecutive addresses of one V^T row instead of colliding in two banks.
#pragma unroll
        for (int t = 0; t < NV; t++) {
            const int v = min(tid + t * AT_THREADS, vmax);
            kr[t] = *reinterpret_cast<const u32x4_t*>(kbase + (size_t)(v / VPR) * HD + (v % VPR) * EPV);
            const int w = min(tid + t * AT_THREADS, AT_CHUNK * VPR - 1);
            vr[t] = *reinterpret_cast<const u32x4_t*>(vbase + (size_t)min(w % AT_CHUNK, n - 1) * HD + (w / AT_CHUNK) * EPV);
        }
#pragma unroll
        for (int t = 0; t < NV; t++) {
            const int v = tid + t * AT_THREADS;
            if (v < AT_CHUNK * VPR) {
                const int pos = v / VPR, d0 = (v % VPR) * EPV;
                const int vpos = v % AT_CHUNK, vd0 = (v / AT_CHUNK) * EPV;
                // positions past the chunk: zero keys and values
                const u32x4_t kk = v <= vmax ? kr[t] : u32x4_t{0u, 0u, 0u, 0u};
                const u32x4_t vv = vpos < n ? vr[t] : u32x4_t{0u, 0u, 0u, 0u};
                if constexpr (F32) {
                    const unsigned kw[4] = {kk.x, kk.y, kk.z, kk.w}, vw[4] = {vv.x, vv.y, vv.z, vv.w};
                    unsigned kh[4], kl[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const float x = __uint_as_float(kw[e]);
                        kh[e] = f32_to_bf16_bits(x);
                        kl[e] = f32_to_bf16_bits(x - bf16_bits_to_f32(kh[e]));
                        const float y = __uint_as_float(vw[e]);
                        const uint16_t yh = f32_to_bf16_bits(y);
                        *reinterpret_cast<uint16_t*>(vT + (vd0 + e) * AM_VPITCH + vpos * 2) = yh;
                        *reinterpret_cast<uint16_t*>(vT + VPLANE + (vd0 + e) * AM_VPITCH + vpos * 2) =
                            f32_to_bf16_bits(y - bf16_bits_to_f32(yh));
                    }
                    *reinterpret_cast<uint2*>(ktile + pos * ROWB + d0 * 2) = make_uint2(kh[0] | (kh[1] << 16), kh[2] | (kh[3] << 16));
                    *reinterpret_cast<uint2*>(ktile + KPLANE + pos * ROWB + d0 * 2) = make_uint2(kl[0] | (kl[1] << 16), kl[2] | (kl[3] << 16));
                } else {
                    *reinterpret_cast<u32x4_t*>(ktile + pos * ROWB + d0 * 2) = kk;
                    const unsigned w4[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        *reinterpret_cast<uint16_t*>(vT + (vd0 + e) * AM_VPITCH + vpos * 2) = (uint16_t)(w4[e >> 1] >> ((e & 1) * 16));
                }
            }
        }
    }
    const float scale = 1.0f / sqrtf((float)HD);
    {   // one group of 16 query vectors per block: the groups of a head run side by side on different CUs instead of
        // one after the other, each re-staging the chunk out of the cache
#pragma unroll
        for (int t = 0; t < QPT; t++) {   // rows past nq: zero queries (their results are never stored)
            const int e = tid + t * AT_THREADS;
            qs[e] = e / HD < nq ? qreg[t] * scale : 0.f;
        }
        __syncthreads();   // K, V^T and the query vectors are staged
        if (n > 0) {
            // phase A: scores.  Wave w takes position tiles w, w + 4; D: lane (c = position, g) holds queries 4g .. 4g+3
            u32x4_t qh[KSTEPS], ql[KSTEPS];
#pragma unroll
            for (int st = 0; st < KSTEPS; st++) split8<F16>(qs + r16 * HD + st * 32 + g * 8, qh[st], ql[st]);
            for (int pt = wave; pt < PT; pt += 4) {
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int st = 0; st < KSTEPS; st++) {
                    const unsigned char* kp = ktile + (pt * 16 + r16) * ROWB + (st * 32 + g * 8) * 2;
                    const u32x4_t kf = *reinterpret_cast<const u32x4_t*>(kp);
                    acc = mfma_h16<F16>(qh[st], kf, acc);
                    acc = mfma_h16<F16>(ql[st], kf, acc);
                    if constexpr (F32) acc = mfma_h16<F16>(qh[st], *reinterpret_cast<const u32x4_t*>(kp + KPLANE), acc);
                }
#pragma unroll
                for (int jx = 0; jx < 4; jx++) sc[(g * 4 + jx) * AT_CHUNK + pt * 16 + r16] = acc[jx];
            }
        }
        __syncthreads();
        // phase B: causal mask, max, exp, sum.  Wave w owns queries 4w .. 4w+3, one per 16-lane row, so the two
        // reductions are DPP row operations; entries past the visible range (and rows past nq) become 0
        {
            const int qi = wave * 4 + g;
            int vis = 0;
            if (qi < nq) vis = min(n, p0 + (q0 + qi) / G + 1 - j0);   // positions of this chunk the row may see
            float sv[AT_CHUNK / 16];
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < AT_CHUNK / 16; t++) {
                const int j = r16 + 16 * t;
                sv[t] = sc[qi * AT_CHUNK + j];
                if (j < vis) mx = fmaxf(mx, sv[t]);
            }
            mx = row16_max(mx);
            float ls = 0.f;
#pragma unroll
            for (int t = 0; t < AT_CHUNK / 16; t++) {
                const int j = r16 + 16 * t;
                const float e = j < vis ? __expf(sv[t] - mx) : 0.f;
                sc[qi * AT_CHUNK + j] = e;
                ls += e;
            }
            ls = row16_sum(ls);
            if (r16 == 0) { ml[qi * 2] = mx; ml[qi * 2 + 1] = ls; }
        }
        __syncthreads();
        // phase C: O = P.V.  Wave w takes output dim tiles w, w + 4, ...; A: lane (r = query, g) holds P[r][32 s + 8g ..],
        // B: lane (c = dim, g) holds V^T[dim][32 s + 8g ..]; D: lane (c = dim, g) holds queries 4g .. 4g+3
        u32x4_t ph[PS], pl[PS];
#pragma unroll
        for (int st = 0; st < PS; st++) split8<F16>(sc + r16 * AT_CHUNK + st * 32 + g * 8, ph[st], pl[st]);
#pragma unroll
        for (int t = 0; t < DTW; t++) {
            const int dt = wave + 4 * t;
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
            if (n > 0) {
#pragma unroll
                for (int st = 0; st < PS; st++) {
                    const unsigned char* vp = vT + (dt * 16 + r16) * AM_VPITCH + (st * 32 + g * 8) * 2;
                    const u32x4_t vf = *reinterpret_cast<const u32x4_t*>(vp);
                    acc = mfma_h16<F16>(ph[st], vf, acc);
                    acc = mfma_h16<F16>(pl[st], vf, acc);
                    if constexpr (F32) acc = mfma_h16<F16>(ph[st], *reinterpret_cast<const u32x4_t*>(vp + VPLANE), acc);
                }
            }
            // the tile goes back through LDS (the query buffer is free by now) so that the block can write whole
            // rows: scattered 4-byte stores straight from the D layout kept every block waiting on the write path
#pragma unroll
            for (int jx = 0; jx < 4; jx++) qs[(g * 4 + jx) * HD + dt * 16 + r16] = acc[jx];
        }
        __syncthreads();
        for (int f = tid; f < nq * (HD / 4); f += AT_THREADS) {
            const int qi = f / (HD / 4), dd = (f % (HD / 4)) * 4;
            const float4 o = *reinterpret_cast<const float4*>(qs + qi * HD + dd);
            const int qg = q0 + qi, r = qg / G, head = kvh * G + qg % G;
            const float mx = ml[qi * 2], ls = ml[qi * 2 + 1];
            if (n_splits == 1) {
                const size_t oo = (size_t)r * dq + (size_t)head * HD + dd;
                const float inv = 1.0f / ls;
                if (out_hi) {
                    split_store(o.x * inv, out_hi, out_lo, oo, out_f16); split_store(o.y * inv, out_hi, out_lo, oo + 1, out_f16);
                    split_store(o.z * inv, out_hi, out_lo, oo + 2, out_f16); split_store(o.w * inv, out_hi, out_lo, oo + 3, out_f16);
                } else {
                    *reinterpret_cast<float4*>(outp + oo) = make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
                }
            } else {
                float* mine = part + (((size_t)r * H + head) * n_splits + split) * (HD + 4);
                *reinterpret_cast<float4*>(mine + dd) = o;
                if (dd == 0) { mine[HD] = n > 0 ? mx : -INFINITY; mine[HD + 1] = n > 0 ? ls : 0.f; }
            }
        }
    }
}

// ---- prompt passes: one block per KV head and 64 query vectors walks the whole causal range -----------------
// Four waves of 16 query vectors each share the staged K / V^T chunks (64 positions at a time, the same 16-bit
// planes as above); a wave keeps its 16 x HD output tile and the running maximum / sum of every query vector in
// registers and rescales them chunk by chunk (online soft-max), so that nothing is written but the finished
// output: no partials, no fold kernel, and a chunk is staged once per 64 query vectors instead of once per 16.
// Layouts as in the kernel above: scores D = lane (c = position, g) holds queries 4g .. 4g+3; output tile D = lane
// (c = dim, g) holds the same queries, so the rescale factors of a lane's queries apply to both.  The exponentials
// cross from the first layout to the A operand of P.V through a wave-private LDS tile.
constexpr int AP_Q = 64;                 // query vectors per block
constexpr int AP_C = 64;                 // cache positions per step
constexpr int AP_VPITCH = AP_C * 2 + 16; // bytes per row of the transposed V tile

template <typename KT, int HD>
static constexpr size_t attn_prompt_lds_bytes()
{
    return (sizeof(KT) == 4 ? 2 : 1) * ((size_t)AP_C * (HD * 2 + 16) + (size_t)HD * AP_VPITCH) + (size_t)4 * 16 * HD * 4;
}

template <typename KT, int HD>
__global__ __launch_bounds__(AT_THREADS) void attn_prompt_kernel(const float* __restrict__ q, int ldq,
                                                                 const KT* __restrict__ kc, const KT* __restrict__ vc,
                                                                 const int* pos_dev, int pos_off, int M, int H, int Hkv,
                                                                 int max_seq, float* __restrict__ outp, int dq,
                                                                 uint16_t* __restrict__ out_hi, uint16_t* __restrict__ out_lo,
                                                                 bool out_f16)
{
    constexpr bool F32 = sizeof(KT) == 4;
    constexpr bool F16 = IsF16<KT>::value;
    constexpr int NP = F32 ? 2 : 1;
    constexpr int ROWB = HD * 2 + 16;
    constexpr int EPV = 16 / (int)sizeof(KT);
    constexpr int VPR = HD / EPV;
    constexpr int KSTEPS = HD / 32;
    constexpr int PT = AP_C / 16;              // position tiles of a chunk (4)
    constexpr int PS = AP_C / 32;              // k-steps of P.V (2)
    constexpr int DT = HD / 16;                // output dim tiles per wave (8 or 4)
    constexpr int KPLANE = AP_C * ROWB, VPLANE = HD * AP_VPITCH;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* ktile = smem;                                       // [NP][AP_C][ROWB]
    unsigned char* vT = smem + NP * KPLANE;                            // [NP][HD][AP_VPITCH]
    float* wbuf = reinterpret_cast<float*>(vT + NP * VPLANE);          // [4 waves][16][HD]: exponentials, then the output tile

    const int kvh = blockIdx.y;
    const int G = H / Hkv, Q = G * M;
    const int p0 = pos_dev[0] + pos_off;
    const int total = p0 + M;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const int q0 = blockIdx.x * AP_Q;
    const int nq = min(AP_Q, Q - q0);
    const int last_vis = p0 + (q0 + nq - 1) / G;          // last position any query vector of the block may see
    float* pw = wbuf + wave * 16 * HD;
    const float scale = 1.0f / sqrtf((float)HD);

    // the wave's 16 query vectors as hi / lo fragments (A operand: lane (r16 = query, g) holds dims 32 st + 8 g ..)
    u32x4_t qh[KSTEPS], ql[KSTEPS];
    {
        const int qv = q0 + min(wave * 16 + r16, nq - 1);      // vectors past nq read a valid one; never stored
        const float* qp = q + (size_t)(qv / G) * ldq + (size_t)(kvh * G + qv % G) * HD;
#pragma unroll
        for (int st = 0; st < KSTEPS; st++) {
            float x[8];
            const float4 a = *reinterpret_cast<const float4*>(qp + st * 32 + g * 8), b = *reinterpret_cast<const float4*>(qp + st * 32 + g * 8 + 4);
            x[0] = a.x * scale; x[1] = a.y * scale; x[2] = a.z * scale; x[3] = a.w * scale;
            x[4] = b.x * scale; x[5] = b.y * scale; x[6] = b.z * scale; x[7] = b.w * scale;
            unsigned h[8], l[8];
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const uint16_t hb = f32_to_h16_bits(x[i], F16);
                h[i] = hb;
                l[i] = f32_to_h16_bits(x[i] - h16_bits_to_f32(hb, F16), F16);
            }
            qh[st] = u32x4_t{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
            ql[st] = u32x4_t{l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
        }
    }
    // causal horizon of the lane's four query vectors (scores layout: queries 4g .. 4g+3 of the wave); -1 = padding
    int horizon[4];
#pragma unroll
    for (int jx = 0; jx < 4; jx++) {
        const int qi = wave * 16 + g * 4 + jx;
        horizon[jx] = qi < nq ? p0 + (q0 + qi) / G : -1;
    }
    float mrun[4], lrun[4];
#pragma unroll
    for (int jx = 0; jx < 4; jx++) { mrun[jx] = -INFINITY; lrun[jx] = 0.f; }
    f32x4_t oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++) oacc[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int j0 = 0; j0 <= last_vis; j0 += AP_C) {
        const int n = min(AP_C, total - j0);               // positions of this chunk that exist (>= 1)
        __syncthreads();                                   // the previous chunk is fully consumed
        {   // stage K (row-major) and V (transposed); every load is issued before the first is used
            const KT* kbase = kc + ((size_t)kvh * max_seq + j0) * HD;
            const KT* vbase = vc + ((size_t)kvh * max_seq + j0) * HD;
            constexpr int NV = AP_C * VPR / AT_THREADS;
            u32x4_t kr[NV], vr[NV];
            const int vmax = n * VPR - 1;
#pragma unroll
            for (int t = 0; t < NV; t++) {
                const int v = min(tid + t * AT_THREADS, vmax);
                kr[t] = *reinterpret_cast<const u32x4_t*>(kbase + (size_t)(v / VPR) * HD + (v % VPR) * EPV);
                const int w = tid + t * AT_THREADS;
                vr[t] = *reinterpret_cast<const u32x4_t*>(vbase + (size_t)min(w % AP_C, n - 1) * HD + (w / AP_C) * EPV);
            }
#pragma unroll
            for (int t = 0; t < NV; t++) {
                const int v = tid + t * AT_THREADS;
                const int pos = v / VPR, d0 = (v % VPR) * EPV;
                const int vpos = v % AP_C, vd0 = (v / AP_C) * EPV;
                const u32x4_t kk = v <= vmax ? kr[t] : u32x4_t{0u, 0u, 0u, 0u};     // positions past the end: zeros
                const u32x4_t vv = vpos < n ? vr[t] : u32x4_t{0u, 0u, 0u, 0u};
                if constexpr (F32) {
                    const unsigned kw[4] = {kk.x, kk.y, kk.z, kk.w}, vw[4] = {vv.x, vv.y, vv.z, vv.w};
                    unsigned kh[4], kl[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const float x = __uint_as_float(kw[e]);
                        kh[e] = f32_to_bf16_bits(x);
                        kl[e] = f32_to_bf16_bits(x - bf16_bits_to_f32(kh[e]));
                        const float y = __uint_as_float(vw[e]);
                        const uint16_t yh = f32_to_bf16_bits(y);
                        *reinterpret_cast<uint16_t*>(vT + (vd0 + e) * AP_VPITCH + vpos * 2) = yh;
                        *reinterpret_cast<uint16_t*>(vT + VPLANE + (vd0 + e) * AP_VPITCH + vpos * 2) =
                            f32_to_bf16_bits(y - bf16_bits_to_f32(yh));
                    }
                    *reinterpret_cast<uint2*>(ktile + pos * ROWB + d0 * 2) = make_uint2(kh[0] | (kh[1] << 16), kh[2] | (kh[3] << 16));
                    *reinterpret_cast<uint2*>(ktile + KPLANE + pos * ROWB + d0 * 2) = make_uint2(kl[0] | (kl[1] << 16), kl[2] | (kl[3] << 16));
                } else {
                    *reinterpret_cast<u32x4_t*>(ktile + pos * ROWB + d0 * 2) = kk;
                    const unsigned w4[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        *reinterpret_cast<uint16_t*>(vT + (vd0 + e) * AP_VPITCH + vpos * 2) = (uint16_t)(w4[e >> 1] >> ((e & 1) * 16));
                }
            }
        }
        __syncthreads();
        // scores of the wave's 16 queries against the 64 positions, masked; running maximum
        float sv[PT][4];
        float mnew[4];
#pragma unroll
        for (int jx = 0; jx < 4; jx++) mnew[jx] = mrun[jx];
#pragma unroll
        for (int pt = 0; pt < PT; pt++) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < KSTEPS; st++) {
                const unsigned char* kp = ktile + (pt * 16 + r16) * ROWB + (st * 32 + g * 8) * 2;
                const u32x4_t kf = *reinterpret_cast<const u32x4_t*>(kp);
                acc = mfma_h16<F16>(qh[st], kf, acc);
                acc = mfma_h16<F16>(ql[st], kf, acc);
                if constexpr (F32) acc = mfma_h16<F16>(qh[st], *reinterpret_cast<const u32x4_t*>(kp + KPLANE), acc);
            }
            const int j = j0 + pt * 16 + r16;
#pragma unroll
            for (int jx = 0; jx < 4; jx++) {
                sv[pt][jx] = j <= horizon[jx] ? acc[jx] : -INFINITY;
                mnew[jx] = fmaxf(mnew[jx], sv[pt][jx]);
            }
        }
        float alpha[4], psum[4];
#pragma unroll
        for (int jx = 0; jx < 4; jx++) {
            mnew[jx] = row16_max(mnew[jx]);                              // over the 16 positions a DPP row holds
            alpha[jx] = mrun[jx] > -INFINITY ? __expf(mrun[jx] - mnew[jx]) : 0.f;
            psum[jx] = 0.f;
        }
#pragma unroll
        for (int pt = 0; pt < PT; pt++)
#pragma unroll
            for (int jx = 0; jx < 4; jx++) {
                const float e = sv[pt][jx] > -INFINITY ? __expf(sv[pt][jx] - mnew[jx]) : 0.f;
                psum[jx] += e;
                pw[(g * 4 + jx) * AP_C + pt * 16 + r16] = e;
            }
#pragma unroll
        for (int jx = 0; jx < 4; jx++) {
            lrun[jx] = lrun[jx] * alpha[jx] + row16_sum(psum[jx]);
            mrun[jx] = mnew[jx];
        }
#pragma unroll
        for (int dt = 0; dt < DT; dt++)
#pragma unroll
            for (int jx = 0; jx < 4; jx++) oacc[dt][jx] *= alpha[jx];
        // O += P.V: A = the exponentials (lane (r16 = query, g) holds positions 32 st + 8 g ..), B = V^T fragments
        u32x4_t ph[PS], pl[PS];
#pragma unroll
        for (int st = 0; st < PS; st++) split8<F16>(pw + r16 * AP_C + st * 32 + g * 8, ph[st], pl[st]);
#pragma unroll
        for (int dt = 0; dt < DT; dt++) {
#pragma unroll
            for (int st = 0; st < PS; st++) {
                const unsigned char* vp = vT + (dt * 16 + r16) * AP_VPITCH + (st * 32 + g * 8) * 2;
                const u32x4_t vf = *reinterpret_cast<const u32x4_t*>(vp);
                oacc[dt] = mfma_h16<F16>(ph[st], vf, oacc[dt]);
                oacc[dt] = mfma_h16<F16>(pl[st], vf, oacc[dt]);
                if constexpr (F32) oacc[dt] = mfma_h16<F16>(ph[st], *reinterpret_cast<const u32x4_t*>(vp + VPLANE), oacc[dt]);
            }
        }
    }
    // finished output: tile -> wave-private LDS ([16 queries][HD]) -> whole rows to memory
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int jx = 0; jx < 4; jx++) pw[(g * 4 + jx) * HD + dt * 16 + r16] = oacc[dt][jx] / lrun[jx];
    for (int f = lane; f < 16 * (HD / 4); f += 64) {
        const int qi = f / (HD / 4), dd = (f % (HD / 4)) * 4;
        if (wave * 16 + qi >= nq) continue;
        const float4 o = *reinterpret_cast<const float4*>(pw + qi * HD + dd);
        const int qg = q0 + wave * 16 + qi, r = qg / G, head = kvh * G + qg % G;
        const size_t oo = (size_t)r * dq + (size_t)head * HD + dd;
        if (out_hi) {
            split_store(o.x, out_hi, out_lo, oo, out_f16); split_store(o.y, out_hi, out_lo, oo + 1, out_f16);
            split_store(o.z, out_hi, out_lo, oo + 2, out_f16); split_store(o.w, out_hi, out_lo, oo + 3, out_f16);
        } else {
            *reinterpret_cast<float4*>(outp + oo) = o;
        }
    }
}

template <typename KT, int HD>
static size_t attn_mfma_lds_bytes()
{
    const size_t planes = sizeof(KT) == 4 ? 2 : 1;
    return planes * ((size_t)AT_CHUNK * (HD * 2 + 16) + (size_t)HD * AM_VPITCH) + (size_t)AT_QPASS * HD * 4 +
           (size_t)AT_QPASS * AT_CHUNK * 4 + (size_t)AT_QPASS * 2 * 4;
}

template <typename KT, int HD>
static size_t attn_lds_bytes()
{
    return (size_t)2 * AT_CHUNK * (HD * sizeof(KT) + 16) + (size_t)AT_QPASS * HD * 4 + (size_t)AT_QPASS * AT_CHUNK * 4 +
           (size_t)AT_QPASS * 2 * 4 + (size_t)AT_THREADS * AT_QPASS * 4;
}

// Folds the split partials of one (row, head) into the attention output.  (Folding inside the
// attention kernel by the last-arriving block needs device-scope fences, which on this
// multi-XCD part cost far more than this extra launch.)
template <int HD>
__global__ void attn_combine_kernel(const float* __restrict__ part, int H, int n_splits, float* __restrict__ out, int dq,
                                    uint16_t* __restrict__ out_hi, uint16_t* __restrict__ out_lo, bool f16)
{
    const int head = blockIdx.x, r = blockIdx.y, d = threadIdx.x;
    const float* p = part + ((size_t)r * H + head) * n_splits * (HD + 4);
    float gm = -INFINITY;
    for (int s = 0; s < n_splits; s++) gm = fmaxf(gm, p[(size_t)s * (HD + 4) + HD]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < n_splits; s++) {
        const float* ps = p + (size_t)s * (HD + 4);
        const float l = ps[HD + 1];
        if (l > 0.f) {
            const float w = __expf(ps[HD] - gm);
            num = fmaf(w, ps[d], num);
            den = fmaf(w, l, den);
        }
    }
    const size_t o = (size_t)r * dq + (size_t)head * HD + d;
    if (out_hi) split_store(num / den, out_hi, out_lo, o, f16);
    else out[o] = num / den;
}

// ---- register-resident variant for few query vectors (decoding, short verification blocks) ----------
// One block = one KV head x one range of positions x up to NQ query vectors.  No LDS staging: a lane
// owns 16 bytes of a cache row (LPP lanes per position, PPL = 64 / LPP positions per wave-wide load)
// and every wave keeps NL such K loads and NL V loads in flight, consecutive waves reading
// consecutive 1 KB pieces.  Scores are reduced over the LPP lanes of a position by shuffles, each wave
// runs an online softmax over its positions, and the NW waves are folded through LDS at the end.  With
// one range per head the block writes the finished output and no second kernel is needed.
template <typename KT> __device__ __forceinline__ void aw_unpack(u32x4_t w, float (&o)[16 / sizeof(KT)]);
template <> __device__ __forceinline__ void aw_unpack<uint16_t>(u32x4_t w, float (&o)[8])
{
    o[0] = __uint_as_float(w.x << 16); o[1] = __uint_as_float(w.x & 0xffff0000u);
    o[2] = __uint_as_float(w.y << 16); o[3] = __uint_as_float(w.y & 0xffff0000u);
    o[4] = __uint_as_float(w.z << 16); o[5] = __uint_as_float(w.z & 0xffff0000u);
    o[6] = __uint_as_float(w.w << 16); o[7] = __uint_as_float(w.w & 0xffff0000u);
}
template <> __device__ __forceinline__ void aw_unpack<f16_t>(u32x4_t w, float (&o)[8])
{
    const f16x8_t h = __builtin_bit_cast(f16x8_t, w);
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] = (float)h[i];
}
template <> __device__ __forceinline__ void aw_unpack<float>(u32x4_t w, float (&o)[4])
{
    o[0] = __uint_as_float(w.x); o[1] = __uint_as_float(w.y); o[2] = __uint_as_float(w.z); o[3] = __uint_as_float(w.w);
}
// sum over the LPP lanes of one position (every lane of the segment gets it).  Segments of 8 and 16
// lanes lie inside one DPP row: rotations by 8, 4, 2, 1 (or a half-row mirror and two quad swaps) add all
// of them without going through the LDS crossbar.
template <int LPP> __device__ __forceinline__ float aw_seg_sum(float v)
{
    if (LPP == 16 || LPP == 32) {
        v = dpp_add<0x128>(v);  // row_ror:8
        v = dpp_add<0x124>(v);  // row_ror:4
        v = dpp_add<0x122>(v);  // row_ror:2
        v = dpp_add<0x121>(v);  // row_ror:1
        if (LPP == 32) v += __shfl_xor(v, 16, 64);
    } else if (LPP == 8) {
        v = dpp_add<0x141>(v);  // row_half_mirror: lane i <- lane 7 - i of its half row
        v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
        v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    } else {
#pragma unroll
        for (int o = LPP / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    }
    return v;
}
// sum / max across the segments of a wave, for values already uniform inside each segment
template <int LPP> __device__ __forceinline__ float aw_xseg_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= LPP; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <int LPP> __device__ __forceinline__ float aw_xseg_max(float v)
{
#pragma unroll
    for (int o = 32; o >= LPP; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

template <typename KT, int HD, int NQ, int NW, int NL>
__global__ __launch_bounds__(NW * 64) void attn_wide_kernel(const float* __restrict__ q, int ldq,
                                                            const KT* __restrict__ kc, const KT* __restrict__ vc,
                                                            const int* pos_dev, int pos_off, int M, int H, int Hkv,
                                                            int max_seq, int n_splits, float* __restrict__ part,
                                                            float* __restrict__ outp, int dq,
                                                            uint16_t* __restrict__ out_hi, uint16_t* __restrict__ out_lo,
                                                            bool out_f16)
{
    constexpr int EPV = 16 / (int)sizeof(KT), LPP = HD / EPV, PPL = 64 / LPP, NT = NW * 64;
    constexpr int PASS = NL * NW * PPL;  // positions one pass of the block covers
    __shared__ __align__(16) float qs[NQ * HD];     // query vectors, pre-scaled
    __shared__ float wacc[NW * NQ * HD];            // per-wave unnormalised outputs
    __shared__ float wml[NW * NQ * 2];              // per-wave (max, sum)
    const int split = blockIdx.x, kvh = blockIdx.y, q0 = blockIdx.z * NQ;
    const int G = H / Hkv, Q = G * M, nq = min(NQ, Q - q0);
    const int p0 = pos_dev[0] + pos_off, total = p0 + M;
    const int chunk = (total + n_splits - 1) / n_splits;
    const int j0 = split * chunk, n = min(chunk, total - j0);  // may be <= 0
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = lane / LPP, sl = (lane % LPP) * EPV;
    const int jlast = j0 + n - 1;
    const int n_pass = n > 0 ? (n + PASS - 1) / PASS : 0;
    const KT* kbase = kc + (size_t)kvh * max_seq * HD + sl;
    const KT* vbase = vc + (size_t)kvh * max_seq * HD + sl;

    u32x4_t kr[NL], vr[NL];
    // addresses are clamped to the last position of the range, never predicated: all loads of a pass stay in
    // flight together, and the positions past the range are masked out of the scores instead
    auto issue_k = [&](int pass) {
#pragma unroll
        for (int t = 0; t < NL; t++) {
            const int j = min(j0 + ((pass * NL + t) * NW + wave) * PPL + seg, jlast);
            kr[t] = *reinterpret_cast<const u32x4_t*>(kbase + (size_t)j * HD);
        }
    };
    auto issue_v = [&](int pass) {
#pragma unroll
        for (int t = 0; t < NL; t++) {
            const int j = min(j0 + ((pass * NL + t) * NW + wave) * PPL + seg, jlast);
            vr[t] = *reinterpret_cast<const u32x4_t*>(vbase + (size_t)j * HD);
        }
    };
    if (n_pass > 0) { issue_k(0); issue_v(0); }

    const float scale = 1.0f / sqrtf((float)HD);
    for (int e = tid; e < NQ * HD; e += NT) {
        const int qi = e / HD;
        float v = 0.f;
        if (qi < nq) {
            const int qg = q0 + qi;
            v = q[(size_t)(qg / G) * ldq + (size_t)(kvh * G + qg % G) * HD + (e % HD)] * scale;
        }
        qs[e] = v;
    }
    int vis[NQ];  // first position a query may NOT see
#pragma unroll
    for (int qi = 0; qi < NQ; qi++) vis[qi] = qi < nq ? min(p0 + (q0 + qi) / G + 1, j0 + n) : j0;
    __syncthreads();

    float m[NQ], l[NQ], acc[NQ][EPV];
#pragma unroll
    for (int qi = 0; qi < NQ; qi++) {
        m[qi] = -INFINITY; l[qi] = 0.f;
#pragma unroll
        for (int u = 0; u < EPV; u++) acc[qi][u] = 0.f;
    }
    for (int pass = 0; pass < n_pass; pass++) {
        float sc[NQ][NL];
#pragma unroll
        for (int t = 0; t < NL; t++) {
            float kf[EPV];
            aw_unpack<KT>(kr[t], kf);
            const int j = j0 + ((pass * NL + t) * NW + wave) * PPL + seg;
#pragma unroll
            for (int qi = 0; qi < NQ; qi++) {
                const float* qv = qs + qi * HD + sl;
                float dot = 0.f;
#pragma unroll
                for (int u = 0; u < EPV; u += 4) {
                    const float4 t4 = *reinterpret_cast<const float4*>(qv + u);
                    dot = fmaf(kf[u], t4.x, dot); dot = fmaf(kf[u + 1], t4.y, dot);
                    dot = fmaf(kf[u + 2], t4.z, dot); dot = fmaf(kf[u + 3], t4.w, dot);
                }
                dot = aw_seg_sum<LPP>(dot);
                sc[qi][t] = j < vis[qi] ? dot : -INFINITY;
            }
        }
        if (pass + 1 < n_pass) issue_k(pass + 1);
#pragma unroll
        for (int qi = 0; qi < NQ; qi++) {
            float mx = sc[qi][0];
#pragma unroll
            for (int t = 1; t < NL; t++) mx = fmaxf(mx, sc[qi][t]);
            mx = aw_xseg_max<LPP>(mx);
            const float mn = fmaxf(m[qi], mx);          // uniform over the wave
            const bool live = mn > -INFINITY;
            const float c = live ? __expf(m[qi] - mn) : 1.0f;   // exp(-inf) = 0 on the first live pass
            l[qi] *= c;
#pragma unroll
            for (int u = 0; u < EPV; u++) acc[qi][u] *= c;
            m[qi] = mn;
#pragma unroll
            for (int t = 0; t < NL; t++) {
                const float e = live ? __expf(sc[qi][t] - mn) : 0.f;  // masked scores give 0
                sc[qi][t] = e;
                l[qi] += e;
            }
        }
#pragma unroll
        for (int t = 0; t < NL; t++) {
            float vf[EPV];
            aw_unpack<KT>(vr[t], vf);
#pragma unroll
            for (int qi = 0; qi < NQ; qi++)
#pragma unroll
                for (int u = 0; u < EPV; u++) acc[qi][u] = fmaf(sc[qi][t], vf[u], acc[qi][u]);
        }
        if (pass + 1 < n_pass) issue_v(pass + 1);
    }
    // fold the position segments of the wave, then the waves of the block
#pragma unroll
    for (int qi = 0; qi < NQ; qi++) {
        l[qi] = aw_xseg_sum<LPP>(l[qi]);
#pragma unroll
        for (int u = 0; u < EPV; u++) acc[qi][u] = aw_xseg_sum<LPP>(acc[qi][u]);
        if (seg == 0) {
#pragma unroll
            for (int u = 0; u < EPV; u++) wacc[(wave * NQ + qi) * HD + sl + u] = acc[qi][u];
        }
        if (lane == 0) { wml[(wave * NQ + qi) * 2] = m[qi]; wml[(wave * NQ + qi) * 2 + 1] = l[qi]; }
    }
    __syncthreads();
    for (int e = tid; e < nq * HD; e += NT) {
        const int qi = e / HD, d = e % HD;
        float gm = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; w++) gm = fmaxf(gm, wml[(w * NQ + qi) * 2]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < NW; w++) {
            const float mw = wml[(w * NQ + qi) * 2];
            if (mw > -INFINITY) {
                const float c = __expf(mw - gm);
                num = fmaf(c, wacc[(w * NQ + qi) * HD + d], num);
                den = fmaf(c, wml[(w * NQ + qi) * 2 + 1], den);
            }
        }
        const int qg = q0 + qi, r = qg / G, head = kvh * G + qg % G;
        if (n_splits == 1) {
            const size_t oo = (size_t)r * dq + (size_t)head * HD + d;
            if (out_hi) split_store(num / den, out_hi, out_lo, oo, out_f16);
            else outp[oo] = num / den;
        } else {
            float* mine = part + (((size_t)r * H + head) * n_splits + split) * (HD + 4);
            mine[d] = num;
            if (d == 0) { mine[HD] = gm; mine[HD + 1] = den; }
        }
    }
}

// Launch plan.  Few query vectors per KV head (Q = M x group size <= AW_MAXQ_TOTAL): the register-resident
// kernel over ranges of about AW_RANGE positions -- a single CU pulls only a few tens of GB/s, so a head's
// cache is spread over many blocks even though that costs the fold of the partial results.  Many query
// vectors (prompt blocks, wide GQA groups): the LDS-staged kernel, which fetches K/V once for all of them.
constexpr int AW_MAXQ_TOTAL = 4;
constexpr int AW_MAX_ROWS = 8;
constexpr int AW_RANGE = 128;
constexpr int AW_MAX_RANGES = 16;
struct AttnPlan { bool wide; int n_splits; bool defer_fold; };

static AttnPlan attn_plan(const Dims& D, int ctx, int M)
{
    const int force_splits = D.opt ? D.opt->attn_splits : 0, force_kernel = D.opt ? D.opt->attn_kernel : 0;
    AttnPlan pl;
    pl.defer_fold = false;
    const int Q = (D.H / D.Hkv) * M;
    // More than 4 query vectors per KV head: the MFMA form of the LDS-staged kernel (12.9 us against 14.5 us at 5 rows,
    // 7B shape, 16-bit cache, fold included).  A model with fp32 WEIGHTS stays in fp32 arithmetic throughout: there a
    // few rows with 1, 2, 4 or 8 query heads per KV head run the register-resident kernel, one block per row and range
    // serving the row's group of heads (two blocks for a group of 8), re-reading a range's K/V from the cache.
    const int G = D.H / D.Hkv;
    pl.wide = Q <= AW_MAXQ_TOTAL ||
              (D.kt == WT_F32 && D.wt == WT_F32 && (G == 1 || G == 2 || G == 4 || G == 8) && M <= AW_MAX_ROWS);
    if (force_kernel == 1 || force_kernel == 3) pl.wide = false;
    if (pl.wide) {
        // ranges of AW_RANGE positions (one pass of the narrowest block shape), at most AW_MAX_RANGES of them; an fp32
        // cache has twice the bytes per position, so its ranges are shorter (more blocks pulling from the cache)
        int ns = ceil_div(ctx, D.kt == WT_F32 ? AW_RANGE * 5 / 8 : AW_RANGE);
        // single row: up to 4 K positions, ranges grow rather than exceed what the output projection folds itself
        // (a longer range costs the attention kernel about 1 us, a separate fold launch 5)
        if (M == 1 && ns > GV_FOLD_MAX && ctx <= GV_FOLD_MAX * 512) ns = GV_FOLD_MAX;
        if (ns > AW_MAX_RANGES) ns = AW_MAX_RANGES;
        if (force_splits > 0) ns = force_splits;
        if (ns > ctx) ns = ctx;
        pl.n_splits = ns;
    } else {
        const int need = ceil_div(ctx, AT_CHUNK);  // a block owns at most AT_CHUNK positions
        pl.n_splits = force_splits > need ? force_splits : need;
    }
    return pl;
}

int attention_splits(const Dims& D, int ctx, int M)
{
    const AttnPlan pl = attn_plan(D, ctx, M);
    return pl.wide ? -pl.n_splits : pl.n_splits;  // distinct values for distinct launch shapes
}

size_t attention_scratch_floats(const Dims& D, int max_rows)
{
    size_t splits = (size_t)ceil_div(D.max_seq, AT_CHUNK);
    if (splits < 64) splits = 64;  // room for the tuning hook
    return (size_t)max_rows * D.H * splits * (D.hd + 4);
}

template <typename KT, int HD, int NQ, int NW, int NL>
static void launch_attn_wide(const Dims& D, const float* q, int ldq, const void* kc, const void* vc, const int* pos_dev,
                             int pos_off, int n_splits, int zq, int M, float* part, float* out, uint16_t* out_hi,
                             uint16_t* out_lo, hipStream_t s)
{
    hipLaunchKernelGGL((attn_wide_kernel<KT, HD, NQ, NW, NL>), dim3(n_splits, D.Hkv, zq), dim3(NW * 64), 0, s, q, ldq,
                       (const KT*)kc, (const KT*)vc, pos_dev, pos_off, M, D.H, D.Hkv, D.max_seq, n_splits, part, out, D.dq,
                       out_hi, out_lo, D.wt == WT_F16);
}

// LDS-staged kernel: MFMA form for 16-bit caches, plain form for fp32 caches
template <typename KT, int HD>
static void launch_attn_staged(const Dims& D, const float* q, int ldq, const void* kc, const void* vc, const int* pos_dev,
                               int pos_off, int n_splits, int M, float* part, float* out, uint16_t* out_hi, uint16_t* out_lo,
                               hipStream_t s)
{
    {
        // MFMA form: 16-bit caches always; fp32 caches when the model's weights are 16-bit (its hi/lo planes carry 16
        // mantissa bits, the precision the multi-row path of such a model works at anyway; an fp32 model keeps fp32)
        if (!(D.opt && D.opt->attn_kernel == 3) && (sizeof(KT) == 2 || D.wt != WT_F32)) {
            const size_t lds = attn_mfma_lds_bytes<KT, HD>();
            static std::atomic<size_t> lds_limit{0};  // per instantiation
            if (ensure_lds((const void*)attn_mfma_kernel<KT, HD>, lds, lds_limit) != hipSuccess)
                return;   // the launch below then fails and reports
            const int Q = (D.H / D.Hkv) * M;
            hipLaunchKernelGGL((attn_mfma_kernel<KT, HD>), dim3(n_splits, D.Hkv, ceil_div(Q, AT_QPASS)), dim3(AT_THREADS), lds, s, q, ldq,
                               (const KT*)kc, (const KT*)vc, pos_dev, pos_off, M, D.H, D.Hkv, D.max_seq, n_splits, part, out, D.dq,
                               out_hi, out_lo, D.wt == WT_F16);
            return;
        }
    }
    const size_t lds = attn_lds_bytes<KT, HD>();
    static std::atomic<size_t> lds_limit{0};  // per instantiation
    if (ensure_lds((const void*)attn_kernel<KT, HD>, lds, lds_limit) != hipSuccess) return;
    hipLaunchKernelGGL((attn_kernel<KT, HD>), dim3(n_splits, D.Hkv, 1), dim3(AT_THREADS), lds, s, q, ldq, (const KT*)kc,
                       (const KT*)vc, pos_dev, pos_off, M, D.H, D.Hkv, D.max_seq, n_splits, part, out, D.dq, out_hi, out_lo,
                       D.wt == WT_F16);
}

template <typename KT, int HD>
static hipError_t attention_t(const Dims& D, const float* q, int ldq, const void* kc, const void* vc, const int* pos_dev,
                              int pos_off, AttnPlan pl, int ctx, int M, float* part, float* out, uint16_t* out_hi,
                              uint16_t* out_lo, hipStream_t s)
{
    const int n_splits = pl.n_splits;
    if (n_splits < 1 || (n_splits > 64 && n_splits > ceil_div(D.max_seq, AT_CHUNK))) return hipErrorInvalidValue;
    // prompt passes (more than 16 rows) of models with 16-bit weights: one kernel over the whole causal range, where
    // it has blocks for a quarter of the CUs at least or the range is short (a block walks the range chunk by chunk:
    // 64 rows behind 640 cached positions take 62 us in 32 blocks, 40 us through the split kernel and its fold)
    if (M > 16 && !pl.wide && (sizeof(KT) == 2 || D.wt != WT_F32) && !(D.opt && D.opt->attn_kernel) &&
        (ceil_div((D.H / D.Hkv) * M, AP_Q) * D.Hkv >= 64 || ctx <= 4 * AP_C)) {
        constexpr size_t lds = attn_prompt_lds_bytes<KT, HD>();
        static std::atomic<size_t> lds_limit{0};  // per instantiation
        hipError_t e = ensure_lds((const void*)attn_prompt_kernel<KT, HD>, lds, lds_limit);
        if (e != hipSuccess) return e;
        const int Q = (D.H / D.Hkv) * M;
        hipLaunchKernelGGL((attn_prompt_kernel<KT, HD>), dim3(ceil_div(Q, AP_Q), D.Hkv), dim3(AT_THREADS), lds, s, q, ldq, (const KT*)kc,
                           (const KT*)vc, pos_dev, pos_off, M, D.H, D.Hkv, D.max_seq, out, D.dq, out_hi, out_lo, D.wt == WT_F16);
        return hipGetLastError();
    }
    if (pl.wide) {
        int Q = (D.H / D.Hkv) * M, zq = 1;
        if (Q > AW_MAXQ_TOTAL) {  // one block per row (its group of heads, or half of a group of 8) and range
            const int G = D.H / D.Hkv;
            Q = G > 4 ? 4 : G;
            zq = M * (G / Q);
        }
        const int span = ceil_div(ctx, n_splits) * (HD / (16 / (int)sizeof(KT)));  // lanes' worth of 16-byte vectors per range
        if (Q == 1 && span <= 8 * 64 * 4) launch_attn_wide<KT, HD, 1, 8, 4>(D, q, ldq, kc, vc, pos_dev, pos_off, n_splits, zq, M, part, out, out_hi, out_lo, s);
        else if (Q == 1 && span <= 16 * 64 * 4) launch_attn_wide<KT, HD, 1, 16, 4>(D, q, ldq, kc, vc, pos_dev, pos_off, n_splits, zq, M, part, out, out_hi, out_lo, s);
        else if (Q == 1) launch_attn_wide<KT, HD, 1, 8, 16>(D, q, ldq, kc, vc, pos_dev, pos_off, n_splits, zq, M, part, out, out_hi, out_lo, s);
        else if (Q == 2) launch_attn_wide<KT, HD, 2, 16, 4>(D, q, ldq, kc, vc, pos_dev, pos_off, n_splits, zq, M, part, out, out_hi, out_lo, s);
        else if (span <= 8 * 64 * 4) launch_attn_wide<KT, HD, 4, 8, 4>(D, q, ldq, kc, vc, pos_dev, pos_off, n_splits, zq, M, part, out, out_hi, out_lo, s);
        else launch_attn_wide<KT, HD, 4, 8, 8>(D, q, ldq, kc, vc, pos_dev, pos_off, n_splits, zq, M, part, out, out_hi, out_lo, s);
    } else {
        launch_attn_staged<KT, HD>(D, q, ldq, kc, vc, pos_dev, pos_off, n_splits, M, part, out, out_hi, out_lo, s);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_splits == 1 || pl.defer_fold) return e;
    hipLaunchKernelGGL((attn_combine_kernel<HD>), dim3(D.H, M), dim3(HD), 0, s, part, D.H, n_splits, out, D.dq, out_hi,
                       out_lo, D.wt == WT_F16);
    return hipGetLastError();
}

hipError_t attention(const Dims& D, const float* q, int ldq, const void* kc, const void* vc, const int* pos_dev,
                     int pos_off, int pos_host_hint, int M, float* part, float* out, uint16_t* out_hi, uint16_t* out_lo,
                     hipStream_t s, int* deferred_splits)
{
    int ctx = pos_host_hint + pos_off + M;  // positions the last row sees
    if (ctx < 1 || ctx > D.max_seq || M < 1) return hipErrorInvalidValue;
    AttnPlan pl = attn_plan(D, ctx, M);
    if (deferred_splits) {  // single row: the consumer (gemv_resid_attn) folds the partials itself
        if (M != 1) return hipErrorInvalidValue;
        pl.defer_fold = pl.n_splits > 1 && pl.n_splits <= GV_FOLD_MAX;
        *deferred_splits = pl.defer_fold ? pl.n_splits : 0;
    }
    if (D.kt == WT_BF16) {
        if (D.hd == 128) return attention_t<uint16_t, 128>(D, q, ldq, kc, vc, pos_dev, pos_off, pl, ctx, M, part, out, out_hi, out_lo, s);
        if (D.hd == 64) return attention_t<uint16_t, 64>(D, q, ldq, kc, vc, pos_dev, pos_off, pl, ctx, M, part, out, out_hi, out_lo, s);
    } else if (D.kt == WT_F16) {
        if (D.hd == 128) return attention_t<f16_t, 128>(D, q, ldq, kc, vc, pos_dev, pos_off, pl, ctx, M, part, out, out_hi, out_lo, s);
        if (D.hd == 64) return attention_t<f16_t, 64>(D, q, ldq, kc, vc, pos_dev, pos_off, pl, ctx, M, part, out, out_hi, out_lo, s);
    } else {
        if (D.hd == 128) return attention_t<float, 128>(D, q, ldq, kc, vc, pos_dev, pos_off, pl, ctx, M, part, out, out_hi, out_lo, s);
        if (D.hd == 64) return attention_t<float, 64>(D, q, ldq, kc, vc, pos_dev, pos_off, pl, ctx, M, part, out, out_hi, out_lo, s);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------
// vocabulary reduction: arg-max, softmax max-probability, entropy confidence (Eq. 1-4)
// ---------------------------------------------------------------------------------------------
constexpr int VR_THREADS = 1024;

__global__ __launch_bounds__(VR_THREADS) void vocab_reduce_kernel(const float* __restrict__ logits, int V, float clamp,
                                                                  float eps, int32_t* tok_out, int tok_stride,
                                                                  int32_t* argmax_out, float* maxprob_out, float* conf_out)
{
    __shared__ float rv[16];
    __shared__ int ri[16];
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* z = logits + (size_t)r * V;
    // pass 1: max and its lowest index
    float m = -INFINITY;
    int mi = 0x7fffffff;
    for (int i = tid; i < V; i += VR_THREADS) {
        float v = fminf(fmaxf(z[i], -clamp), clamp);
        if (v > m) { m = v; mi = i; }  // ascending i per thread: first occurrence kept
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float om = __shfl_xor(m, o, 64);
        int oi = __shfl_xor(mi, o, 64);
        if (om > m || (om == m && oi < mi)) { m = om; mi = oi; }
    }
    if (lane == 0) { rv[wave] = m; ri[wave] = mi; }
    __syncthreads();
    m = rv[0]; mi = ri[0];
#pragma unroll
    for (int w = 1; w < 16; w++) {
        float om = rv[w]; int oi = ri[w];
        if (om > m || (om == m && oi < mi)) { m = om; mi = oi; }
    }
    // pass 2: Z = sum exp(z - m)
    float zs = 0.f;
    for (int i = tid; i < V; i += VR_THREADS) zs += expf(fminf(fmaxf(z[i], -clamp), clamp) - m);
    float Z = block_sum<16>(zs, rv);
    if (tid == 0) {
        if (tok_out) tok_out[(size_t)r * tok_stride] = mi;
        if (argmax_out) argmax_out[r] = mi;
        if (maxprob_out) maxprob_out[r] = 1.0f / Z;
    }
    if (conf_out) {
        // pass 3: H = -sum p log(p + eps)
        float hs = 0.f;
        const float invZ = 1.0f / Z;
        for (int i = tid; i < V; i += VR_THREADS) {
            float pr = expf(fminf(fmaxf(z[i], -clamp), clamp) - m) * invZ;
            hs -= pr * logf(pr + eps);
        }
        float Hs = block_sum<16>(hs, rv);
        if (tid == 0) conf_out[r] = 1.0f - Hs / logf((float)V);
    }
}

// means[t] = mean over p < n_pos of v[p * n_taps + t], summed in position order (one thread per tap row)
__global__ void window_mean_kernel(const float* __restrict__ v, int n_pos, int n_taps, float* __restrict__ means)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_taps) return;
    float s = 0.f;
    for (int p = 0; p < n_pos; p++) s += v[(size_t)p * n_taps + t];
    means[t] = s / (float)n_pos;
}
hipError_t window_mean(const float* v, int n_pos, int n_taps, float* means, hipStream_t s)
{
    if (n_pos < 1 || n_taps < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(window_mean_kernel, dim3(ceil_div(n_taps, 64)), dim3(64), 0, s, v, n_pos, n_taps, means);
    return hipGetLastError();
}

hipError_t vocab_reduce(const float* logits, int M, int V, float clamp, float eps, int32_t* tok_out, int tok_stride,
                        int32_t* argmax_out, float* maxprob_out, float* conf_out, hipStream_t s)
{
    hipLaunchKernelGGL(vocab_reduce_kernel, dim3(M), dim3(VR_THREADS), 0, s, logits, V, clamp, eps, tok_out, tok_stride,
                       argmax_out, maxprob_out, conf_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// static scratch (for the entry point that allocates nothing)
// ---------------------------------------------------------------------------------------------
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)12 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

size_t static_scratch_bytes() { return STATIC_SCRATCH_BYTES; }

// `scratch` names the array only in device code; in host code the name is a stand-in, not an address.  The device
// address is asked of the runtime once per device, with that device current, and kept.
hipError_t static_scratch_for_device(int device, void** ptr_out)
{
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void* ptr[MAX_DEV] = {};
    if (!ptr_out || device < 0 || device >= MAX_DEV) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[device] = p;
    }
    *ptr_out = ptr[device];
    return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// state kernels
// ---------------------------------------------------------------------------------------------
__global__ void set_state_kernel(int32_t* tok0, int32_t token, int* pos_dev, int pos)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { tok0[0] = token; pos_dev[0] = pos; }
}
hipError_t set_state(int32_t* tok0, int32_t token, int* pos_dev, int pos, hipStream_t s)
{
    hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, s, tok0, token, pos_dev, pos);
    return hipGetLastError();
}

__global__ void advance_state_kernel(int* pos_dev, int delta, int32_t* tok0, const int32_t* src)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        pos_dev[0] += delta;
        if (src) tok0[0] = src[0];
    }
}
hipError_t advance_state(int* pos_dev, int delta, int32_t* tok0, const int32_t* src, hipStream_t s)
{
    hipLaunchKernelGGL(advance_state_kernel, dim3(1), dim3(64), 0, s, pos_dev, delta, tok0, src);
    return hipGetLastError();
}

template <typename KT>
__global__ void kv_poison_kernel(KT* kv, int planes, int max_seq, int hd, const int* pos_dev)
{
    // kv: [planes][max_seq][hd] where planes = L * 2 * Hkv
    const int from = pos_dev[0];
    size_t per_plane = (size_t)(max_seq - from) * hd;
    size_t total = per_plane * planes;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        size_t pl = i / per_plane, o = i % per_plane;
        Elem<KT>::put(kv, (pl * max_seq + from) * hd + o, __int_as_float(0x7fc00000));
    }
}
hipError_t kv_poison(const Dims& D, void* kv_all, const int* pos_dev, hipStream_t s)
{
    int planes = D.L * 2 * D.Hkv;
    if (D.kt == WT_BF16)
        hipLaunchKernelGGL(kv_poison_kernel<uint16_t>, dim3(1024), dim3(256), 0, s, (uint16_t*)kv_all, planes, D.max_seq,
                           D.hd, pos_dev);
    else if (D.kt == WT_F16)
        hipLaunchKernelGGL(kv_poison_kernel<f16_t>, dim3(1024), dim3(256), 0, s, (f16_t*)kv_all, planes, D.max_seq, D.hd,
                           pos_dev);
    else
        hipLaunchKernelGGL(kv_poison_kernel<float>, dim3(1024), dim3(256), 0, s, (float*)kv_all, planes, D.max_seq, D.hd,
                           pos_dev);
    return hipGetLastError();
}

__global__ void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}
hipError_t copy_f32(const float* src, float* dst, size_t n, hipStream_t s)
{
    int blocks = (int)((n + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks), dim3(256), 0, s, src, dst, n);
    return hipGetLastError();
}

// Read-only streaming probe: every lane keeps eight non-temporal 128-bit loads in flight (the access shape of the
// weight-streaming kernels, minus their arithmetic); a wave reads 1 KB contiguous per load instruction.
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4_t* __restrict__ src, size_t n_vec, float* sink)
{
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 7 * stride < n_vec; i += 8 * stride) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n_vec; i += stride) {
        const u32x4_t a = __builtin_nontemporal_load(src + i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) sink[0] = 1.0f;  // practically never true; keeps the loads alive
}
hipError_t read_probe(const void* dev, size_t bytes, float* sink_dev, hipStream_t s)
{
    hipLaunchKernelGGL(read_probe_kernel, dim3(256 * 8), dim3(256), 0, s, (const u32x4_t*)dev, bytes / 16, sink_dev);
    return hipGetLastError();
}

}  // namespace ssdk
