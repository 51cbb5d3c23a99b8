// Traffic-matrix construction (paper Section 5 "Integration into MoE systems"):
// MoE frameworks all-gather the per-expert token counts before every dispatch, so
// every rank holds counts[src][e] = tokens GPU src routes to expert e; the
// GPU-to-GPU byte matrix that the scheduler consumes is
//     traffic[src][h] = token_bytes * sum over experts e placed on GPU h of counts[src][e].
// One workgroup per (matrix, source GPU): the row of counts is read once
// (coalesced), accumulated per destination GPU in LDS (integer atomics,
// order-independent) and the traffic row written once: HBM-bound,
// 8*N*E bytes read + 8*N*N bytes written per matrix.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"

namespace fastk {

constexpr int BT_THREADS = 256;

// status[b]: 0, or -1 if a count is negative or an expert is placed outside
// 0..N-1 (zeroed by bt_zero before; merged with atomic min)
__global__ void __launch_bounds__(256) bt_zero(int32_t* __restrict__ status, int B) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B) status[i] = 0;
}

__global__ void __launch_bounds__(BT_THREADS)
bt_build(const i64* __restrict__ counts, const int32_t* __restrict__ expert_to_gpu,
         i64* __restrict__ traffic, int32_t* __restrict__ status, int N, int E, i64 token_bytes) {
    extern __shared__ __align__(16) unsigned char bt_smem[];
    u64* acc = reinterpret_cast<u64*>(bt_smem);          // [N]
    __shared__ int bad;
    const int src = blockIdx.x;
    const int b = blockIdx.y;
    const int tid = threadIdx.x;
    for (int h = tid; h < N; h += BT_THREADS) acc[h] = 0;
    if (tid == 0) bad = 0;
    __syncthreads();
    const i64* row = counts + ((size_t)b * N + src) * E;
    const int32_t* place = expert_to_gpu + (size_t)b * E;
    bool err = false;
    for (int e = tid; e < E; e += BT_THREADS) {
        const i64 c = row[e];
        const int h = place[e];
        if (c < 0 || h < 0 || h >= N) err = true;
        else if (c != 0) atomicAdd(&acc[h], (u64)c);
    }
    if (err) bad = 1;
    __syncthreads();
    i64* out = traffic + ((size_t)b * N + src) * N;
    for (int h = tid; h < N; h += BT_THREADS) out[h] = (i64)acc[h] * token_bytes;
    if (tid == 0 && bad) atomicMin(&status[b], -1);
}

}  // namespace fastk
