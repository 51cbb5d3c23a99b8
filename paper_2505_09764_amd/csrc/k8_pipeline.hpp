// Completion time of the overlapped pipeline (paper Section 4.3 "Pipeline
// structure", Fig. 7): balancing first; then the scale-out stages back to back;
// the intra-server portion on the scale-up fabric alongside the first stage;
// stage i's redistribution starts when its scale-out has ended and the scale-up
// fabric is free, overlapping the following stages; the last redistribution is
// exposed.  Every step that moves bytes costs the wake-up delay plus
// bytes / bandwidth (Section 5.4).
//
// With out = end of the latest scale-out and up = time the scale-up fabric becomes
// free, one stage (scale-out time x, redistribution time y) is the map
//   out' = out + x,   up' = max(out + x, up) + y
// which is linear in the (max, +) semiring: out' = out + A, up' = max(out + C, up + D)
// with (A, C, D) = (x, x + y, y), and maps compose as
//   (A1, C1, D1) then (A2, C2, D2) = (A1 + A2, max(A1 + C2, C1 + D2), D1 + D2).
// So the K dependent steps become a reduction: every thread composes a contiguous
// run of stages, thread 0 composes the 256 partial maps in order.  One workgroup
// per matrix; the stage weights and the two scale-up volumes of a matrix come from the
// caller's summary buffers (pl_summary copies them out of the plan's workspace).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"

namespace fastk {

constexpr int PL_THREADS = 256;

// grid (ceil(max_stages / 256) + 1, B): the stage weights of matrix b, copied as they are
// (entries >= K hold whatever an earlier call left), and, by the last block of the row, the
// largest balancing and intra-server volumes over the servers' records.
__global__ void __launch_bounds__(PL_THREADS)
pl_summary(const i64* __restrict__ wsPart, const i64* __restrict__ wsC, i64* __restrict__ out_weight,
           i64* __restrict__ out_volume, int S, int max_stages) {
    const int b = blockIdx.y;
    const int tid = threadIdx.x;
    if (blockIdx.x + 1 < gridDim.x) {
        const int s = blockIdx.x * PL_THREADS + tid;
        if (s < max_stages) out_weight[(size_t)b * max_stages + s] = wsC[(size_t)b * max_stages + s];
        return;
    }
    __shared__ i64 sBal[PL_THREADS / 64], sIntra[PL_THREADS / 64];
    i64 bal = 0, intra = 0;
    for (int a = tid; a < S; a += PL_THREADS) {
        const i64* part = wsPart + ((size_t)b * S + a) * K1_PART;
        bal = max(bal, part[0]);
        intra = max(intra, part[1]);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        bal = max(bal, __shfl_xor(bal, o, 64));
        intra = max(intra, __shfl_xor(intra, o, 64));
    }
    if ((tid & 63) == 0) { sBal[tid >> 6] = bal; sIntra[tid >> 6] = intra; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < PL_THREADS / 64; ++w) {
            bal = max(bal, sBal[w]);
            intra = max(intra, sIntra[w]);
        }
        out_volume[(size_t)b * 2] = bal;
        out_volume[(size_t)b * 2 + 1] = intra;
    }
}

__global__ void __launch_bounds__(PL_THREADS)
pl_time(const i64* __restrict__ weight, const i64* __restrict__ volume,
        const int32_t* __restrict__ num_stages, const int32_t* __restrict__ order,
        const i64* __restrict__ redis, double* __restrict__ out_time, int G, int max_stages,
        double bw_up, double bw_out, double delay) {
    __shared__ double sA[PL_THREADS], sC[PL_THREADS], sD[PL_THREADS];
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int K = min(num_stages[b], max_stages);     // a count beyond the capacity is not trusted
    double* out = out_time + (size_t)b * 2;
    if (K < 0) {
        if (tid < 2) out[tid] = 0.0;
        return;
    }
    const i64 bal = volume[(size_t)b * 2], intra = volume[(size_t)b * 2 + 1];

    const i64* c = weight + (size_t)b * max_stages;
    const int32_t* ord = order ? order + (size_t)b * max_stages : nullptr;
    const i64* rb = redis ? redis + (size_t)b * max_stages : nullptr;
    const int per = (K + PL_THREADS - 1) / PL_THREADS;
    const int e0 = tid * per;
    const int e1 = min(K, e0 + per);
    double A = 0.0, C = -INFINITY, D = 0.0;
    for (int e = e0; e < e1; ++e) {
        int s = ord ? ord[e] : e;
        if (s < 0 || s >= K) s = e;                     // not a stage index: keep memory safe
        const i64 l = c[s];
        const i64 v = rb ? rb[s] : (i64)(G - 1) * l;
        const double x = delay + (double)l / bw_out;
        A = A + x;
        if (v > 0) {
            const double y = delay + (double)v / bw_up;
            C = fmax(A, C) + y;                         // A already includes x
            D = D + y;
        }
    }
    sA[tid] = A;
    sC[tid] = C;
    sD[tid] = D;
    __syncthreads();
    if (tid == 0) {
        double tA = 0.0, tC = -INFINITY, tD = 0.0;
        for (int t = 0; t < PL_THREADS; ++t) {
            const double a2 = sA[t], c2 = sC[t], d2 = sD[t];
            tC = fmax(tA + c2, tC + d2);
            tA = tA + a2;
            tD = tD + d2;
        }
        double t0 = 0.0;
        if (bal > 0) t0 = delay + (double)bal / bw_up;
        double up0 = t0;
        if (intra > 0) up0 = t0 + (delay + (double)intra / bw_up);
        const double out_end = t0 + tA;
        const double up = fmax(t0 + tC, up0 + tD);
        out[0] = fmax(out_end, up);
        out[1] = out_end;
    }
}

}  // namespace fastk
