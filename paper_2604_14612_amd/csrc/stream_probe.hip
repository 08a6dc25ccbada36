// Streaming-rate probe for the weight-streaming kernels (stand-alone, read-only, every access in bounds).
//
// Reads one N x K bf16 matrix (22016 x 4096: the gate/up matrices of the 7B shape, 180 MB, twelve cold copies per
// timing) with the access shapes the GEMV / MFMA kernels could use and prints the time per pass, launch included:
//   rows R x S KB   a wave owns R rows and has S KB of each in flight (a load instruction = 1 KB of one row)
//   half rows       a wave owns 16 rows, an instruction covers 2 rows x 512 bytes
//   fragments       the MFMA A-operand shape: an instruction covers 16 rows x 64 bytes
//   gemv variants   the rows 2 x 4 shape plus the arithmetic of a GEMV (input vector in LDS, 8 FMAs per load, wave
//                   reduction), with the LDS vector in natural order (lanes 32 bytes apart: two-way bank conflicts),
//                   in two planes (conflict-free), from registers (no LDS in the loop), and with four rows per wave
// Usage: stream_probe   (no arguments)
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("%s: %s\n", #x, hipGetErrorString(e_)); std::exit(1); } } while (0)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 ldnt(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
__device__ __forceinline__ uint32_t fold(u32x4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

// RR rows x SS KB of each row in flight per wave.  Needs N % RR == 0 and K % (SS * 512) == 0.
template <int RR, int SS>
__global__ __launch_bounds__(512) void probe_rows(const uint16_t* w, int N, int K, uint32_t* sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwaves = gridDim.x * 8, gw = blockIdx.x * 8 + wave;
    uint32_t acc = 0;
    for (int r0 = gw * RR; r0 + RR - 1 < N; r0 += nwaves * RR) {
        for (int k0 = 0; k0 < K; k0 += SS * 512) {
            u32x4 v[RR][SS];
#pragma unroll
            for (int r = 0; r < RR; r++)
#pragma unroll
                for (int s = 0; s < SS; s++) v[r][s] = ldnt(w + (size_t)(r0 + r) * K + k0 + s * 512 + lane * 8);
#pragma unroll
            for (int r = 0; r < RR; r++)
#pragma unroll
                for (int s = 0; s < SS; s++) acc ^= fold(v[r][s]);
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;   // keeps the loads alive
}

// 16 rows per wave; lane l reads 16 bytes of row 2 q + (l >> 5) at byte 16 (l & 31): an instruction covers 2 rows x
// 512 contiguous bytes, 8 instructions 16 rows x 256 k; DD such groups in flight.  Needs N % 16 == 0, K % (DD * 256) == 0.
template <int DD>
__global__ __launch_bounds__(512) void probe_half(const uint16_t* w, int N, int K, uint32_t* sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwaves = gridDim.x * 8, gw = blockIdx.x * 8 + wave;
    uint32_t acc = 0;
    for (int r0 = gw * 16; r0 + 15 < N; r0 += nwaves * 16) {
        const uint16_t* base = w + (size_t)(r0 + (lane >> 5)) * K + (lane & 31) * 8;
        for (int k0 = 0; k0 < K; k0 += DD * 256) {
            u32x4 v[DD][8];
#pragma unroll
            for (int s = 0; s < DD; s++)
#pragma unroll
                for (int q = 0; q < 8; q++) v[s][q] = ldnt(base + (size_t)(2 * q) * K + k0 + s * 256);
#pragma unroll
            for (int s = 0; s < DD; s++)
#pragma unroll
                for (int q = 0; q < 8; q++) acc ^= fold(v[s][q]);
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

// MFMA A-operand shape: lane (i = lane % 16, g = lane / 16) reads 16 bytes of row i at k0 + 32 s + 8 g; DD k-steps
// in flight.  Needs N % 16 == 0, K % (DD * 32) == 0.
template <int DD>
__global__ __launch_bounds__(512) void probe_frag(const uint16_t* w, int N, int K, uint32_t* sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int nwaves = gridDim.x * 8, gw = blockIdx.x * 8 + wave;
    uint32_t acc = 0;
    for (int r0 = gw * 16; r0 + 15 < N; r0 += nwaves * 16) {
        const uint16_t* row = w + (size_t)(r0 + i) * K + g * 8;
        for (int k0 = 0; k0 < K; k0 += DD * 32) {
            u32x4 v[DD];
#pragma unroll
            for (int s = 0; s < DD; s++) v[s] = ldnt(row + k0 + s * 32);
#pragma unroll
            for (int s = 0; s < DD; s++) acc ^= fold(v[s]);
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

// rows shape + GEMV arithmetic.  MODE 0: x from registers (no LDS in the loop); 1: x in LDS in natural order;
// 2: x in LDS in two planes (conflict-free); 3: as 2 with four rows x 2 KB per wave.  K * 4 bytes of dynamic LDS.
template <int MODE>
__global__ __launch_bounds__(512) void probe_gemv(const uint16_t* w, const float* x, float* y, int N, int K)
{
    extern __shared__ float xs[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nwaves = gridDim.x * 8, gw = blockIdx.x * 8 + wave;
    constexpr int R = MODE == 3 ? 4 : 2, S = MODE == 3 ? 2 : 4;
    for (int i = threadIdx.x; i < K; i += 512) {
        const int c = i >> 9, e = i & 511, l = e >> 3, j = e & 7;
        xs[MODE >= 2 ? c * 512 + (j >> 2) * 256 + l * 4 + (j & 3) : i] = x[i];
    }
    __syncthreads();
    const float4 cx = *reinterpret_cast<const float4*>(xs + lane * 4);
    for (int r0 = gw * R; r0 + R - 1 < N; r0 += nwaves * R) {
        float acc[R];
#pragma unroll
        for (int r = 0; r < R; r++) acc[r] = 0.f;
        for (int k0 = 0; k0 < K; k0 += S * 512) {
            u32x4 v[R][S];
#pragma unroll
            for (int r = 0; r < R; r++)
#pragma unroll
                for (int s = 0; s < S; s++) v[r][s] = ldnt(w + (size_t)(r0 + r) * K + k0 + s * 512 + lane * 8);
#pragma unroll
            for (int s = 0; s < S; s++) {
                float4 xa, xb;
                if (MODE == 0) { xa = cx; xb = cx; }
                else if (MODE == 1) {
                    xa = *reinterpret_cast<const float4*>(xs + k0 + s * 512 + lane * 8);
                    xb = *reinterpret_cast<const float4*>(xs + k0 + s * 512 + lane * 8 + 4);
                } else {
                    xa = *reinterpret_cast<const float4*>(xs + k0 + s * 512 + lane * 4);
                    xb = *reinterpret_cast<const float4*>(xs + k0 + s * 512 + 256 + lane * 4);
                }
#pragma unroll
                for (int r = 0; r < R; r++) {
                    const u32x4 q = v[r][s];
                    acc[r] += __uint_as_float(q.x << 16) * xa.x + __uint_as_float(q.x & 0xffff0000u) * xa.y +
                              __uint_as_float(q.y << 16) * xa.z + __uint_as_float(q.y & 0xffff0000u) * xa.w +
                              __uint_as_float(q.z << 16) * xb.x + __uint_as_float(q.z & 0xffff0000u) * xb.y +
                              __uint_as_float(q.w << 16) * xb.z + __uint_as_float(q.w & 0xffff0000u) * xb.w;
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; r++) {
            float t = acc[r];
            for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, 64);
            if (lane == 0) y[r0 + r] = t;
        }
    }
}

int main()
{
    const int N = 22016, K = 4096, COPIES = 12;   // N % 16 == 0, K % 4096 == 0: every shape above stays in bounds
    const size_t elems = (size_t)N * K;
    uint16_t* w; uint32_t* sink; float *x, *y;
    CK(hipMalloc(&x, K * 4)); CK(hipMalloc(&y, N * 4)); CK(hipMemset(x, 0, K * 4));
    CK(hipMalloc(&w, elems * 2 * COPIES)); CK(hipMalloc(&sink, 64));
    CK(hipMemset(w, 1, elems * 2 * COPIES));
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    auto run = [&](const char* name, auto launch) {
        float best = 1e30f;
        for (int rep = 0; rep < 4; rep++) {
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(a, 0));
            for (int c = 0; c < COPIES; c++) launch(w + (size_t)c * elems);
            CK(hipEventRecord(b, 0)); CK(hipEventSynchronize(b));
            float ms; CK(hipEventElapsedTime(&ms, a, b));
            if (ms < best) best = ms;
        }
        CK(hipGetLastError());
        const double us = best * 1e3 / COPIES;
        std::printf("  %-58s %8.2f us  %7.0f GB/s\n", name, us, elems * 2.0 / us / 1e3);
        std::fflush(stdout);
    };
#define ROWS(RR, SS, label) run(label, [&](const uint16_t* p) { hipLaunchKernelGGL((probe_rows<RR, SS>), dim3(blocks), dim3(512), 0, 0, p, N, K, sink); })
#define GEMV(MODE, label) run(label, [&](const uint16_t* p) { hipLaunchKernelGGL((probe_gemv<MODE>), dim3(blocks), dim3(512), K * 4, 0, p, x, y, N, K); })
    for (int blocks : {256, 512, 768}) {
        std::printf("-- %d blocks of 8 waves, %d x %d bf16 (%.1f MB)\n", blocks, N, K, elems * 2.0 / 1e6);
        ROWS(2, 4, "rows 2 x 4 KB in flight per wave (the GEMV's shape)");
        ROWS(1, 8, "rows 1 x 8 KB");
        ROWS(2, 2, "rows 2 x 2 KB");
        ROWS(2, 1, "rows 2 x 1 KB");
        ROWS(4, 2, "rows 4 x 2 KB");
        ROWS(4, 1, "rows 4 x 1 KB");
        ROWS(8, 1, "rows 8 x 1 KB");
        run("half rows: 16 rows x 512 B per 8 instructions, 1 group", [&](const uint16_t* p) { hipLaunchKernelGGL(probe_half<1>, dim3(blocks), dim3(512), 0, 0, p, N, K, sink); });
        run("half rows: 16 rows x 512 B per 8 instructions, 2 groups", [&](const uint16_t* p) { hipLaunchKernelGGL(probe_half<2>, dim3(blocks), dim3(512), 0, 0, p, N, K, sink); });
        run("fragments: 16 rows x 64 B per instruction, 4 in flight", [&](const uint16_t* p) { hipLaunchKernelGGL(probe_frag<4>, dim3(blocks), dim3(512), 0, 0, p, N, K, sink); });
        run("fragments: 16 rows x 64 B per instruction, 8 in flight", [&](const uint16_t* p) { hipLaunchKernelGGL(probe_frag<8>, dim3(blocks), dim3(512), 0, 0, p, N, K, sink); });
        run("fragments: 16 rows x 64 B per instruction, 16 in flight", [&](const uint16_t* p) { hipLaunchKernelGGL(probe_frag<16>, dim3(blocks), dim3(512), 0, 0, p, N, K, sink); });
        GEMV(0, "gemv: rows 2 x 4 + FMAs, x from registers");
        GEMV(1, "gemv: rows 2 x 4 + FMAs, x in LDS, natural order");
        GEMV(2, "gemv: rows 2 x 4 + FMAs, x in LDS, two planes");
        GEMV(3, "gemv: rows 4 x 2 + FMAs, x in LDS, two planes");
    }
    return 0;
}
