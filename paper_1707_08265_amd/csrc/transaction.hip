// Key of a transaction (Sec. 4.1 of the Dragon paper): a function -- here: the result of pruning one graph for
// one choice of target sets -- is bound to a hashing key generated from that choice, so that asking for it again
// builds nothing new.  The paper names no hash; the key used here is a 128-bit digest of the target sets as
// dgn_prune receives them, the word sequence
//     w = [ num_sets, n, rowptr[0..n], idx[0..m-1] ]
// with  digest_k = sum_i mix((i + 1) * G + w_i * C_k + S_k)  mod 2^64  for k = 0, 1, where mix is the output
// function of SplitMix64 (Steele, Lea, Flood, OOPSLA 2014) and G its increment.  A sum of position-keyed terms
// has no order, so every thread adds up the terms of the words it happens to hold: two launches (partial sums
// per workgroup, then their sum), no atomics, nothing to clear.
#include "common.h"

namespace dgn {

constexpr u64 kGolden = 0x9E3779B97F4A7C15ull;
constexpr u64 kMulA = 0xC2B2AE3D27D4EB4Full, kAddA = 0x165667B19E3779F9ull;
constexpr u64 kMulB = 0xD6E8FEB86659FD93ull, kAddB = 0x27D4EB2F165667C5ull;

__device__ __forceinline__ u64 splitmix_out(u64 z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ u64 wave_sum64(u64 v)
{
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) v += shfl_xor64(v, d);
    return v;
}

// partial[2 * block + k] = sum of this workgroup's terms of half k
__global__ __launch_bounds__(256) void k_digest_partial(int32_t num_sets, int64_t n, const int32_t *tgt_rowptr,
                                                         int64_t num_targets, const int32_t *tgt_idx, u64 *partial)
{
    __shared__ u64 s_sum[2][4];
    const int64_t words = 2 + (n + 1) + num_targets;
    const int64_t gsize = (int64_t)gridDim.x * blockDim.x;
    u64 a = 0, b = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += gsize) {
        int32_t w;
        if (i == 0) w = num_sets;
        else if (i == 1) w = (int32_t)n;
        else if (i < 3 + n) w = tgt_rowptr[i - 2];
        else w = tgt_idx[i - 3 - n];
        const u64 key = (u64)(i + 1) * kGolden, v = (u64)(uint32_t)w;
        a += splitmix_out(key + v * kMulA + kAddA);
        b += splitmix_out(key + v * kMulB + kAddB);
    }
    a = wave_sum64(a);
    b = wave_sum64(b);
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    if (lane == 0) { s_sum[0][wave] = a; s_sum[1][wave] = b; }
    __syncthreads();
    if (threadIdx.x < 2)
        partial[2 * blockIdx.x + threadIdx.x] = s_sum[threadIdx.x][0] + s_sum[threadIdx.x][1] + s_sum[threadIdx.x][2] +
                                                s_sum[threadIdx.x][3];
}

// out[k] = sum of the partial sums of half k (one wave)
__global__ __launch_bounds__(64) void k_digest_total(const u64 *partial, int blocks, u64 *out)
{
    u64 a = 0, b = 0;
    for (int i = lane_id(); i < blocks; i += kWave) {
        a += partial[2 * i];
        b += partial[2 * i + 1];
    }
    a = wave_sum64(a);
    b = wave_sum64(b);
    if (lane_id() == 0) { out[0] = a; out[1] = b; }
}

size_t digest_scratch_bytes() { return (size_t)(kDigestMaxBlocks + 1) * 2 * sizeof(u64); }

hipError_t launch_target_digest(int32_t num_sets, int64_t n, const int32_t *tgt_rowptr, int64_t num_targets,
                                const int32_t *tgt_idx, void *scratch, u64 **digest_dev, hipStream_t s)
{
    const int64_t words = 2 + (n + 1) + num_targets;
    int64_t blocks = (words + 255) / 256;
    if (blocks > kDigestMaxBlocks) blocks = kDigestMaxBlocks;
    u64 *partial = static_cast<u64 *>(scratch);
    u64 *out = partial + 2 * kDigestMaxBlocks;
    hipLaunchKernelGGL(k_digest_partial, dim3((unsigned)blocks), dim3(256), 0, s, num_sets, n, tgt_rowptr, num_targets,
                       tgt_idx, partial);
    hipLaunchKernelGGL(k_digest_total, dim3(1), dim3(64), 0, s, partial, (int)blocks, out);
    *digest_dev = out;
    return hipGetLastError();
}

}  // namespace dgn
