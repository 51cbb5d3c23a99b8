// Execution order of the stages (paper Appendix, proof of Theorem 2): the stages
// of a plan are executed in ascending order of their transfer size, which is
// what lets each stage's redistribution hide under the next stage and what the
// completion-time model assumes.  order[b][.] lists the stage indices of matrix b
// by ascending weight (largest per-lane byte count of the stage), equal weights
// in extraction order.
//
// so_weights reads the stage rows once (HBM-bound, 8*S bytes per stage): one
// wavefront per stage row, wave maximum, and writes (weight, index) keys padded
// to a power of two with +infinity keys.  so_sort is a bitonic sort of those
// keys by (weight, index) - a total order, so the result does not depend on the
// sorting network - with one workgroup per matrix: chunks of 4096 keys are sorted and
// merged in LDS, only the steps that pair elements of different chunks touch the
// global (L2-resident) arrays.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"

namespace fastk {

constexpr int SO_THREADS = 1024;
constexpr int SO_W_THREADS = 256;

// grid (ceil(P / 4), B): each of the 4 wavefronts of a workgroup takes one key slot
__global__ void __launch_bounds__(SO_W_THREADS)
so_weights(const i64* __restrict__ stage_bytes, const int32_t* __restrict__ num_stages,
           u64* __restrict__ keys, int32_t* __restrict__ idx, int S, int max_stages, int P) {
    const int b = blockIdx.y;
    const int s = blockIdx.x * (SO_W_THREADS / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (s >= P) return;
    const int K = min(num_stages[b], max_stages);     // a count beyond the capacity is not trusted
    u64 key = ~0ull;
    if (s < K) {
        const i64* row = stage_bytes + ((size_t)b * max_stages + s) * S;
        i64 m = 0;
        for (int a = lane; a < S; a += 64) m = max(m, row[a]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = max(m, __shfl_xor(m, off, 64));
        key = (u64)m;
    }
    if (lane == 0) {
        keys[(size_t)b * P + s] = key;
        idx[(size_t)b * P + s] = s;
    }
}

constexpr int SO_CHUNK = 4096;     // keys sorted in LDS at a time (48 KiB)

// One compare-exchange step of the bitonic network on (key, index) pairs: element t against
// its partner t ^ j, ascending where (t & kk) == 0.  (key, index) is a total order, so the
// result does not depend on the network.
__device__ __forceinline__ bool so_out_of_order(u64 ka, int32_t ia, u64 kb, int32_t ib, bool up) {
    const bool a_after_b = ka > kb || (ka == kb && ia > ib);
    return a_after_b == up;
}

// grid (B), 1024 threads.  The steps whose partner distance is below SO_CHUNK run on chunks
// held in LDS (all of them for n <= SO_CHUNK); only the few steps with a larger distance go
// through the global (L2-resident) arrays.
__global__ void __launch_bounds__(SO_THREADS)
so_sort(u64* __restrict__ keys, int32_t* __restrict__ idx, const int32_t* __restrict__ num_stages,
        int32_t* __restrict__ order, int max_stages, int P) {
    __shared__ u64 lk[SO_CHUNK];
    __shared__ int32_t li[SO_CHUNK];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int K = min(num_stages[b], max_stages);     // a count beyond the capacity is not trusted
    if (K <= 0) return;
    u64* k = keys + (size_t)b * P;
    int32_t* x = idx + (size_t)b * P;
    // sort only the smallest power of two that holds the K real keys
    int n = 1;
    while (n < K) n <<= 1;
    const int ch = n < SO_CHUNK ? n : SO_CHUNK;
    // steps (kk, j) for j = jhi, jhi/2, ..., 1 on every chunk, in LDS; kk_lo..kk_hi when the
    // chunk is sorted from scratch
    auto local_steps = [&](int kk_lo, int kk_hi, int jhi) {
        for (int c0 = 0; c0 < n; c0 += ch) {
            for (int t = tid; t < ch; t += SO_THREADS) { lk[t] = k[c0 + t]; li[t] = x[c0 + t]; }
            __syncthreads();
            for (int kk = kk_lo; kk <= kk_hi; kk <<= 1)
                for (int j = (kk >> 1) < jhi ? (kk >> 1) : jhi; j > 0; j >>= 1) {
                    for (int t = tid; t < ch; t += SO_THREADS) {
                        const int p = t ^ j;
                        if (p > t) {
                            const u64 ka = lk[t], kb = lk[p];
                            const int32_t ia = li[t], ib = li[p];
                            if (so_out_of_order(ka, ia, kb, ib, ((c0 + t) & kk) == 0)) {
                                lk[t] = kb; lk[p] = ka;
                                li[t] = ib; li[p] = ia;
                            }
                        }
                    }
                    __syncthreads();
                }
            for (int t = tid; t < ch; t += SO_THREADS) { k[c0 + t] = lk[t]; x[c0 + t] = li[t]; }
            __syncthreads();
        }
    };
    local_steps(2, ch, ch >> 1);                       // every chunk sorted (alternating direction)
    for (int kk = ch << 1; kk <= n; kk <<= 1) {
        for (int j = kk >> 1; j >= ch; j >>= 1) {       // partners in different chunks
            for (int t = tid; t < n; t += SO_THREADS) {
                const int p = t ^ j;
                if (p > t) {
                    const u64 ka = k[t], kb = k[p];
                    const int32_t ia = x[t], ib = x[p];
                    if (so_out_of_order(ka, ia, kb, ib, (t & kk) == 0)) {
                        k[t] = kb; k[p] = ka;
                        x[t] = ib; x[p] = ia;
                    }
                }
            }
            __syncthreads();
        }
        local_steps(kk, kk, ch >> 1);
    }
    int32_t* out = order + (size_t)b * max_stages;
    for (int s = tid; s < K; s += SO_THREADS) out[s] = x[s];
}

}  // namespace fastk
