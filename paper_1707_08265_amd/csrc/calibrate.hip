// Machine rates that bound the traversal of Algorithm 1 on this chip (dgn_calibrate, declared in dgn.h).
//
// The frontier traversal moves few bytes; what it is made of is random 8-byte reads of masks and adjacency
// records, 64-bit atomic ORs on masks, kernel launches (one per wide level) and, inside a level, a chain of
// accesses that each need the answer of the one before.  None of these has a published peak, so they are
// measured here, on the caller's buffer (the size of the mask array, so that locality is the workload's), with
// HIP events on the caller's stream.
#include <string.h>

#include "common.h"

namespace dgn {

__device__ __forceinline__ u64 cal_mix(u64 z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

enum { kCalLoad = 0, kCalAtomic = 1, kCalStore = 2, kCalAtomicNoReturn = 3, kCalLoadAndAtomic = 4, kCalAtomicRun = 5 };

// `total` independent accesses to words drawn uniformly from A[0, nwords)
template <int MODE>
__global__ __launch_bounds__(256) void k_cal_random(u64 *A, u64 nwords, u64 total, u64 *sink)
{
    const u64 gtid = (u64)blockIdx.x * blockDim.x + threadIdx.x, gsize = (u64)gridDim.x * blockDim.x;
    u64 acc = 0;
    for (u64 i = gtid; i < total; i += gsize) {
        // (kCalAtomicRun: the 64 lanes of a wave hit 64 consecutive words, the run's start is random)
        const u64 idx = MODE == kCalAtomicRun ? ((cal_mix((i >> 6) * 7 + MODE) % (nwords >> 6)) << 6) + (i & 63) : cal_mix(i * 7 + MODE) % nwords;
        if (MODE == kCalLoad) acc += load_coherent(&A[idx]);
        else if (MODE == kCalAtomic) acc += atomicOr(&A[idx], (u64)1 << (i & 63));
        else if (MODE == kCalAtomicNoReturn) atomicOr(&A[idx], (u64)1 << (i & 63));     // result unused: no data comes back
        else if (MODE == kCalAtomicRun) atomicOr(&A[idx], (u64)1 << (i & 63));
        else if (MODE == kCalLoadAndAtomic) {                                            // a load and an atomic, unrelated addresses
            acc += load_coherent(&A[cal_mix(i * 11 + 5) % nwords]);
            atomicOr(&A[idx], (u64)1 << (i & 63));
        }
        else A[idx] = 0;
    }
    if (acc == 0x123456789abcdefull) sink[0] = acc;       // keeps the loads alive
}

// one lane walks `steps` accesses, each address depending on the value the access before returned
template <int MODE>
__global__ void k_cal_chain(u64 *A, u64 nwords, int steps, u64 *sink)
{
    u64 idx = 12345 % nwords, acc = 0;
    for (int i = 0; i < steps; ++i) {
        const u64 v = MODE == kCalLoad ? load_coherent(&A[idx]) : atomicOr(&A[idx], (u64)2);
        acc += v;
        idx = (cal_mix(idx + i) + (v & 1)) % nwords;
    }
    sink[1] = acc;
}

// every wave adds to ONE word: what a single shared counter costs
__global__ __launch_bounds__(256) void k_cal_same_address(u64 *A, u64 *sink)
{
    u64 r = 0;
    if (lane_id() == 0) r = atomicAdd(&A[0], (u64)1);
    if (r == 0xffffffffffffffffull) sink[0] = r;
}

__global__ __launch_bounds__(256) void k_cal_empty(u64 *sink)
{
    if (sink == nullptr && threadIdx.x == 1024) sink[0] = 0;   // never true
}

__global__ __launch_bounds__(256) void k_cal_copy(const ulonglong2 *src, ulonglong2 *dst, u64 n)
{
    const u64 gsize = (u64)gridDim.x * blockDim.x;
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gsize) dst[i] = src[i];
}

// Every wave scan and reduction of common.h on one wave's 64 values (in), side by side (out: five arrays of n)
__global__ __launch_bounds__(256) void k_selftest_wave(const int *in, int *out, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;        // n is a multiple of the block size
    const int v = in[i];
    out[i] = wave_incl_scan(v);
    out[n + i] = wave_incl_max(v);
    out[2 * n + i] = wave_sum(v);
    out[3 * n + i] = wave_max(v);
    const u64 o = wave_or(((u64)(uint32_t)v << 32) | (uint32_t)(v * 0x9E3779B1u));
    // and the three-input bit operation, its middle operand the same for the whole wave as in the sort's ranking
    const uint32_t u = (uint32_t)__builtin_amdgcn_readfirstlane(v) * 0xC2B2AE35u;
    const uint32_t x = or_of_xor((uint32_t)v * 0x85EBCA6Bu, u, (uint32_t)v * 0x27D4EB2Fu);
    out[4 * n + i] = (int)((uint32_t)(o ^ (o >> 32)) ^ x);
}

}  // namespace dgn

using namespace dgn;

extern "C" int dgn_selftest_wave_ops(void *buffer, size_t bytes, dgn_stream stream)
{
    constexpr int kWaves = 64, n = kWaves * kWave;
    if (!buffer) return DGN_ERR_NULL_PTR;
    if (bytes < (size_t)6 * n * sizeof(int) || ((uintptr_t)buffer & 15)) return DGN_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // small sums, large values, sparse values and negative ones, a wave each in turn (a fixed linear congruential sequence)
    static int h_in[n], h_out[5 * n];
    uint32_t x = 12345u;
    for (int i = 0; i < n; ++i) {
        x = x * 1664525u + 1013904223u;
        const int r = (int)(x >> 8), w = i / kWave;
        h_in[i] = w % 4 == 0 ? r % 5 : w % 4 == 1 ? r % 100000 : w % 4 == 2 ? (r % 7 == 0 ? r % 64 : 0) : -(r % 1000) - 1;
    }
    int *d_in = static_cast<int *>(buffer), *d_out = d_in + n;
    if (hipMemcpyAsync(d_in, h_in, sizeof(h_in), hipMemcpyHostToDevice, s) != hipSuccess) return DGN_ERR_HIP;
    hipLaunchKernelGGL(k_selftest_wave, dim3(n / 256), dim3(256), 0, s, d_in, d_out, n);
    if (hipGetLastError() != hipSuccess) return DGN_ERR_HIP;
    if (hipMemcpyAsync(h_out, d_out, sizeof(h_out), hipMemcpyDeviceToHost, s) != hipSuccess) return DGN_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return DGN_ERR_HIP;
    int bad = 0;
    for (int w = 0; w < kWaves; ++w) {
        int tot = 0, top = -2147483647 - 1;
        u64 all = 0;
        for (int l = 0; l < kWave; ++l) {
            const int v = h_in[w * kWave + l];
            tot += v;
            top = top > v ? top : v;
            all |= ((u64)(uint32_t)v << 32) | (uint32_t)(v * 0x9E3779B1u);
        }
        int run = 0, run_max = -2147483647 - 1;
        for (int l = 0; l < kWave; ++l) {
            const int i = w * kWave + l;
            run += h_in[i];
            run_max = run_max > h_in[i] ? run_max : h_in[i];
            bad += h_out[i] != run;
            bad += h_out[n + i] != run_max;
            bad += h_out[2 * n + i] != tot;
            bad += h_out[3 * n + i] != top;
            const uint32_t v = (uint32_t)h_in[i], u = (uint32_t)h_in[w * kWave] * 0xC2B2AE35u;
            const uint32_t x = (v * 0x85EBCA6Bu) | (u ^ (v * 0x27D4EB2Fu));
            bad += h_out[4 * n + i] != (int)((uint32_t)(all ^ (all >> 32)) ^ x);
        }
    }
    return bad;
}

extern "C" int dgn_calibrate(void *buffer, size_t bytes, dgn_machine_rates *out, dgn_stream stream)
{
    if (!buffer || !out) return DGN_ERR_NULL_PTR;
    if (bytes < (size_t)1 << 20 || ((uintptr_t)buffer & 15)) return DGN_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    u64 *A = static_cast<u64 *>(buffer);
    const u64 nwords = (bytes / 8 - 64) & ~(u64)1;          // the last 512 bytes are the kernels' sink
    u64 *sink = A + nwords;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return DGN_ERR_HIP;
    auto timed = [&](auto &&enqueue, int reps) -> float {    // best of `reps` runs, in ms; negative on error
        float best = -1.0f;
        for (int r = 0; r <= reps; ++r) {                    // run 0 warms up
            if (hipEventRecord(e0, s) != hipSuccess) return -1.0f;
            enqueue();
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1.0f;
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.0f;
            if (r > 0 && (best < 0.0f || ms < best)) best = ms;
        }
        return best;
    };
    FillRegion all[1] = {{A, (size_t)(nwords + 64) * 8}};
    if (launch_clear(all, 1, s) != hipSuccess) return DGN_ERR_HIP;
    memset(out, 0, sizeof(*out));
    const u64 total = (u64)1 << 24;
    const dim3 grid(4096), block(256);
    float ms;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_random<kCalLoad>, grid, block, 0, s, A, nwords, total, sink); }, 3);
    out->random_load_gps = ms > 0 ? (float)(total / (ms * 1e6)) : 0.0f;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_random<kCalAtomic>, grid, block, 0, s, A, nwords, total, sink); }, 3);
    out->random_atomic_gps = ms > 0 ? (float)(total / (ms * 1e6)) : 0.0f;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_random<kCalStore>, grid, block, 0, s, A, nwords, total, sink); }, 3);
    out->random_store_gps = ms > 0 ? (float)(total / (ms * 1e6)) : 0.0f;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_random<kCalAtomicNoReturn>, grid, block, 0, s, A, nwords, total, sink); }, 3);
    out->random_atomic_noreturn_gps = ms > 0 ? (float)(total / (ms * 1e6)) : 0.0f;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_random<kCalLoadAndAtomic>, grid, block, 0, s, A, nwords, total, sink); }, 3);
    out->random_load_and_atomic_gps = ms > 0 ? (float)(total / (ms * 1e6)) : 0.0f;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_random<kCalAtomicRun>, grid, block, 0, s, A, nwords, total, sink); }, 3);
    out->run_atomic_gps = ms > 0 ? (float)(total / (ms * 1e6)) : 0.0f;
    const int steps = 2000;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_chain<kCalLoad>, dim3(1), dim3(1), 0, s, A, nwords, steps, sink); }, 2);
    const float empty1 = timed([&] { hipLaunchKernelGGL(k_cal_empty, dim3(1), dim3(64), 0, s, sink); }, 5);
    out->dependent_load_ns = ms > 0 ? (ms - empty1) * 1e6f / steps : 0.0f;
    ms = timed([&] { hipLaunchKernelGGL(k_cal_chain<kCalAtomic>, dim3(1), dim3(1), 0, s, A, nwords, steps, sink); }, 2);
    out->dependent_atomic_ns = ms > 0 ? (ms - empty1) * 1e6f / steps : 0.0f;
    const int same_blocks = 2048;                            // 8192 waves, one atomic each
    ms = timed([&] { hipLaunchKernelGGL(k_cal_same_address, dim3(same_blocks), block, 0, s, A, sink); }, 3);
    const float empty_wide = timed([&] { hipLaunchKernelGGL(k_cal_empty, dim3(2048), block, 0, s, sink); }, 5);
    out->same_address_atomic_ns = ms > 0 ? (ms - empty_wide) * 1e6f / (same_blocks * 4) : 0.0f;
    out->launch_floor_us = empty_wide * 1e3f;
    const int chain = 100;
    ms = timed([&] { for (int i = 0; i < chain; ++i) hipLaunchKernelGGL(k_cal_empty, dim3(2048), block, 0, s, sink); }, 3);
    out->launch_back_to_back_us = ms > 0 ? ms * 1e3f / chain : 0.0f;
    const u64 half = (nwords / 2) & ~(u64)1;                 // copy the first half onto the second
    ms = timed([&] {
        hipLaunchKernelGGL(k_cal_copy, grid, block, 0, s, reinterpret_cast<const ulonglong2 *>(A),
                           reinterpret_cast<ulonglong2 *>(A + half), half / 2);
    }, 3);
    out->copy_gbs = ms > 0 ? (float)(2.0 * half * 8 / (ms * 1e6)) : 0.0f;
    out->buffer_bytes = (int64_t)bytes;
    const hipError_t e = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e == hipSuccess ? DGN_OK : DGN_ERR_HIP;
}
