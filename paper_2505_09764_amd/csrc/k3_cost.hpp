// Kernel 3: analytical two-tier completion time of each plan.
//
// One workgroup per matrix.  Evaluates on the actual plan the four serial terms
// of the paper's completion-time model (Appendix, proof of Theorem 2: balance ->
// intra-server portion -> Birkhoff stages -> last stage's redistribution; each
// term is bytes / bandwidth as in the Section 5.4 simulator, wake-up delay 0) and
// the optimal time of Theorem 1:
//   t0    = max over GPUs of max(bytes handed off, bytes handed in) / B_up
//   t1    = max over GPUs of max(intra-server bytes out, in) / B_up
//   t2    = (sum of stage weights) / B_out
//   t3    = (G-1) * largest stage weight / B_up
//   t_exc = exposed redistribution when B_up < (G-1) B_out: with the stage weights
//           sorted ascending, sum_{i>=1} max(0, (G-1) l_{i-1}/B_up - l_i/B_out)
//           (proof of Theorem 2, steps (i)-(iii)); otherwise 0
//   delay = link wake-up delay, added once per executed step: the balance (if
//           anything is handed off), the intra-server portion (if any), each
//           stage, the last redistribution (if G > 1 and there is a stage)
//   t_opt = max(max row sum, max column sum of T) / (G * B_out)
// All reductions are exact int64; each term is one conversion and one division.
// out[b] = { t0 + t1 + t2 + t3 + t_exc + delay * steps, t0, t2, t_opt }.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"
#include "matching.hpp"

namespace fastk {

constexpr int K3_THREADS = 256;

// Sum or maximum (of non-negative values) over the workgroup, the same in every thread.
template <int THREADS>
__device__ __forceinline__ i64 block_reduce(i64 v, bool is_max, i64* scratch) {
    if (is_max) {
        v = (i64)wave_max_u64((u64)v);           // DPP, result wave-uniform
    } else {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    }
    if constexpr (THREADS == 64) return v;       // one wavefront: every lane holds the result
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[w] = v;
    __syncthreads();
    i64 r = scratch[0];
    for (int k = 1; k < THREADS / 64; ++k) r = is_max ? max(r, scratch[k]) : r + scratch[k];
    return r;
}

// sort_n: 0, or the power of two >= K capacity for which dynamic LDS was provided
// (only when the exposed-redistribution term is needed).
// THREADS = K3_THREADS: a workgroup of its own (tid = threadIdx.x); THREADS = 64: the tail of
// the decomposition kernel's wavefront (tid = lane; sort_n must be 0: no barrier is reached).
template <int THREADS>
__device__ __forceinline__ void
k3_matrix(const i64* __restrict__ wsT, const i64* __restrict__ wsPart, const i64* __restrict__ wsC,
          const int32_t* __restrict__ out_num, double* __restrict__ out_time, int S, int G,
          int max_stages, double bw_up, double bw_out, double delay, int sort_n, int b,
          int tid, unsigned char* k3_smem) {
    __shared__ i64 scratch[K3_THREADS / 64];
    const int K = out_num[b];
    double* out = out_time + (size_t)b * 4;
    if (K < 0) {
        if (tid < 4) out[tid] = 0.0;
        return;
    }
    i64 bal = 0, intra = 0, rowmax = 0, colmax = 0;
    for (int a = tid; a < S; a += THREADS) {
        const i64* part = wsPart + ((size_t)b * S + a) * K1_PART;
        bal = max(bal, part[0]);
        intra = max(intra, part[1]);
        rowmax = max(rowmax, part[3]);
        // column sum of T, eight loads in flight
        const i64* col = wsT + (size_t)b * S * S + a;
        i64 cs = 0;
        int r = 0;
        for (; r + 8 <= S; r += 8) {
            i64 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = col[(size_t)(r + j) * S];
#pragma unroll
            for (int j = 0; j < 8; ++j) cs += v[j];
        }
        for (; r < S; ++r) cs += col[(size_t)r * S];
        colmax = max(colmax, cs);
    }
    i64 csum = 0, cmax = 0;
    const i64* c = wsC + (size_t)b * max_stages;
    {
        int s = tid;
        for (; s + 7 * THREADS < K; s += 8 * THREADS) {
            i64 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = c[s + j * THREADS];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                csum += v[j];
                cmax = max(cmax, v[j]);
            }
        }
        for (; s < K; s += THREADS) {
            const i64 v = c[s];
            csum += v;
            cmax = max(cmax, v);
        }
    }
    bal = block_reduce<THREADS>(bal, true, scratch);
    intra = block_reduce<THREADS>(intra, true, scratch);
    const i64 big = block_reduce<THREADS>(max(rowmax, colmax), true, scratch);
    csum = block_reduce<THREADS>(csum, false, scratch);
    cmax = block_reduce<THREADS>(cmax, true, scratch);

    if (sort_n > 0) {
        // bitonic sort of the stage weights in LDS, padded with the largest value
        i64* l = reinterpret_cast<i64*>(k3_smem);
        for (int s = tid; s < sort_n; s += THREADS) l[s] = s < K ? c[s] : INT64_MAX;
        __syncthreads();
        for (int k = 2; k <= sort_n; k <<= 1)
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int t = tid; t < sort_n; t += THREADS) {
                    const int p = t ^ j;
                    if (p > t) {
                        const i64 x = l[t], y = l[p];
                        const bool up = (t & k) == 0;
                        if ((x > y) == up) { l[t] = y; l[p] = x; }
                    }
                }
                __syncthreads();
            }
    }

    if (tid == 0) {
        const double t0 = (double)bal / bw_up;
        const double t1 = (double)intra / bw_up;
        const double t2 = (double)csum / bw_out;
        const double t3 = (double)((i64)(G - 1) * cmax) / bw_up;
        double texc = 0.0;
        if (sort_n > 0) {
            const i64* l = reinterpret_cast<const i64*>(k3_smem);
            for (int i = 1; i < K; ++i) {
                const double redis = (double)((i64)(G - 1) * l[i - 1]) / bw_up;
                const double next = (double)l[i] / bw_out;
                if (redis > next) texc += redis - next;
            }
        }
        double tp = t0 + t1;
        tp = tp + t2;
        tp = tp + t3;
        tp = tp + texc;
        const int steps = (bal > 0 ? 1 : 0) + (intra > 0 ? 1 : 0) + K +
                          ((i64)(G - 1) * cmax > 0 ? 1 : 0);
        tp = __dadd_rn(tp, __dmul_rn(delay, (double)steps));   // no fused multiply-add
        out[0] = tp;
        out[1] = t0;
        out[2] = t2;
        out[3] = (double)big / ((double)G * bw_out);
    }
}

// One workgroup per matrix: matrix blockIdx.x.  (static: the header is included by more than
// one translation unit of the library.)
static __global__ void __launch_bounds__(K3_THREADS)
k3_cost(const i64* __restrict__ wsT, const i64* __restrict__ wsPart, const i64* __restrict__ wsC,
        const int32_t* __restrict__ out_num, double* __restrict__ out_time, int S, int G,
        int max_stages, double bw_up, double bw_out, double delay, int sort_n) {
    extern __shared__ __align__(16) unsigned char k3_smem[];
    k3_matrix<K3_THREADS>(wsT, wsPart, wsC, out_num, out_time, S, G, max_stages, bw_up, bw_out,
                          delay, sort_n, (int)blockIdx.x, (int)threadIdx.x, k3_smem);
}

}  // namespace fastk
