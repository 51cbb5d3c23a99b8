// Kernels of the SpreadOut baseline (paper Section 4.2 "SpreadOut: one-to-one but
// not optimal"; Section 5.4 compares FAST with it in simulation).
//
// SpreadOut pairs endpoint s with endpoint (s+i) mod n in stage i = 1..n-1; a
// stage lasts as long as its largest transfer, so the completion time is the sum
// over shifted diagonals of the largest entry's transfer time, plus the link
// wake-up delay per non-empty stage.  Two views are evaluated per matrix:
//   [0] over the N GPUs on the raw matrix (a pair inside a server moves at B_up,
//       a pair across servers at B_out);
//   [1] over the S servers on the balanced per-lane matrix Q = ceil(T/G) (FAST's
//       balancing followed by shifted diagonals instead of Birkhoff stages).
//
// spo_scan reads the traffic matrix once (HBM-bound, 8*N*N bytes per matrix): a
// workgroup owns the rows of a few servers, keeps the per-diagonal maxima and its
// servers' tile totals in LDS (integer max / add atomics: order-independent) and
// merges the maxima into the per-matrix arrays with global atomic max.
// spo_finish turns the maxima into times: the per-stage terms are computed in
// parallel, then added in stage order by one thread so that the floating-point
// sum is the same as a sequential evaluation.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"

namespace fastk {

constexpr int SPO_THREADS = 256;

// servers per workgroup of spo_scan
inline int spo_chunk_servers(int S, int G) {
    int cs = 64 / G;
    if (cs < 1) cs = 1;
    return cs > S ? S : cs;
}
inline size_t spo_scan_lds_bytes(int S, int G) {
    const int N = S * G;
    return (size_t)(2 * N + spo_chunk_servers(S, G) * S + 1) * sizeof(i64);
}

__global__ void __launch_bounds__(256) spo_zero(u64* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// wsDiag[b][2][N]: largest intra-server / cross-server entry of every shifted
// diagonal; wsT[b][S][S]: server-to-server totals; wsNeg[b][chunks]: negative flag.
template <int G, bool VEC>
__global__ void __launch_bounds__(SPO_THREADS)
spo_scan(const i64* __restrict__ traffic, u64* __restrict__ wsDiag, i64* __restrict__ wsT,
         int* __restrict__ wsNeg, int S, int CS) {
    extern __shared__ __align__(16) unsigned char spo_smem[];
    const int N = S * G;
    const int b = blockIdx.y;
    const int a0 = blockIdx.x * CS;                      // first server of this chunk
    const int ns = min(CS, S - a0);                      // servers in this chunk
    u64* dup = reinterpret_cast<u64*>(spo_smem);         // [N] intra-server maxima per diagonal
    u64* dout = dup + N;                                 // [N] cross-server maxima
    u64* Tl = dout + N;                                  // [CS][S] tile totals
    u64* flag = Tl + (size_t)CS * S;
    const int tid = threadIdx.x;
    for (int i = tid; i < 2 * N + CS * S + 1; i += SPO_THREADS) dup[i] = 0;
    __syncthreads();

    const i64* mat = traffic + (size_t)b * N * N;
    const int tile_rows = ns * G * S;                    // (row r of the chunk, tile d)
    bool neg = false;
    for (int t = tid; t < tile_rows; t += SPO_THREADS) {
        const int r = t / S;                             // row inside the chunk
        const int d = t - r * S;                         // destination server
        const int al = r / G;                            // server inside the chunk
        const int g = a0 * G + r;                        // sending GPU
        const i64* src = mat + (size_t)g * N + (size_t)d * G;
        i64 v[G];
        if constexpr (VEC) {
            const i64x2* s2 = reinterpret_cast<const i64x2*>(src);
#pragma unroll
            for (int j = 0; j < G / 2; ++j) {
                const i64x2 w = s2[j];
                v[2 * j] = w.x;
                v[2 * j + 1] = w.y;
            }
        } else {
#pragma unroll
            for (int j = 0; j < G; ++j) v[j] = src[j];
        }
        const bool same = d == a0 + al;
        u64* dm = same ? dup : dout;
        int dg = d * G - g;                              // diagonal of column d*G
        if (dg < 0) dg += N;
        i64 sum = 0;
#pragma unroll
        for (int j = 0; j < G; ++j) {
            int x = dg + j;
            x = x >= N ? x - N : x;
            if (x != 0) {                                // x == 0 is the GPU diagonal
                neg |= v[j] < 0;
                sum += v[j];
                if (v[j] > 0) atomicMax(&dm[x], (u64)v[j]);
            }
        }
        if (!same && sum != 0) atomicAdd(&Tl[(size_t)al * S + d], (u64)sum);
    }
    if (neg) *flag = 1;
    __syncthreads();

    u64* gd = wsDiag + (size_t)b * 2 * N;
    for (int i = tid; i < 2 * N; i += SPO_THREADS)
        if (dup[i] != 0) atomicMax(&gd[i], dup[i]);
    for (int i = tid; i < ns * S; i += SPO_THREADS)
        wsT[((size_t)b * S + a0) * S + i] = (i64)Tl[i];
    if (tid == 0) wsNeg[(size_t)b * gridDim.x + blockIdx.x] = (int)*flag;
}

// out[b] = { GPU-level time, server-level time }, or { -1, -1 } for a matrix with
// a negative off-diagonal entry.
__global__ void __launch_bounds__(SPO_THREADS)
spo_finish(const u64* __restrict__ wsDiag, const i64* __restrict__ wsT,
           const int* __restrict__ wsNeg, double* __restrict__ out, int S, int G, int chunks,
           double bw_up, double bw_out, double delay) {
    extern __shared__ __align__(16) unsigned char spo_smem[];
    double* term = reinterpret_cast<double*>(spo_smem);      // [N] then reused for [S]
    __shared__ int bad;
    const int N = S * G;
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    if (tid == 0) bad = 0;
    __syncthreads();
    for (int c = tid; c < chunks; c += SPO_THREADS)
        if (wsNeg[(size_t)b * chunks + c]) bad = 1;
    __syncthreads();
    if (bad) {
        if (tid < 2) out[(size_t)b * 2 + tid] = -1.0;
        return;
    }
    const u64* gd = wsDiag + (size_t)b * 2 * N;
    for (int i = tid; i < N; i += SPO_THREADS) {
        const u64 up = gd[i], ot = gd[N + i];
        double t = 0.0;
        if (i > 0 && (up | ot) != 0) {
            const double x = (double)(i64)up / bw_up, y = (double)(i64)ot / bw_out;
            t = delay + (x > y ? x : y);
        }
        term[i] = t;
    }
    __syncthreads();
    // The terms are added in stage order by one thread (the sum a sequential evaluation gives);
    // empty stages hold 0.0, which leaves a non-negative sum unchanged, so nothing is tested.
    auto ordered_sum = [&](int n) -> double {
        double t = 0.0;
        int i = 1;
        for (; i + 8 <= n; i += 8) {
            double v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = term[i + j];
#pragma unroll
            for (int j = 0; j < 8; ++j) t = t + v[j];
        }
        for (; i < n; ++i) t = t + term[i];
        return t;
    };
    double tg = 0.0;
    if (tid == 0) tg = ordered_sum(N);
    __syncthreads();
    const i64* T = wsT + (size_t)b * S * S;
    for (int i = tid; i < S; i += SPO_THREADS) {
        // largest entry of the shifted diagonal; rounding up after the maximum gives the same
        // value as rounding every entry up first, with one division instead of S
        i64 m = 0;
        if (i > 0) {
            int a = 0;
            for (; a + 8 <= S; a += 8) {
                i64 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    int d = a + j + i;
                    d = d >= S ? d - S : d;
                    v[j] = T[(size_t)(a + j) * S + d];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) m = max(m, v[j]);
            }
            for (; a < S; ++a) {
                int d = a + i;
                d = d >= S ? d - S : d;
                m = max(m, T[(size_t)a * S + d]);
            }
            m = (m + G - 1) / G;
        }
        term[i] = m > 0 ? delay + (double)m / bw_out : 0.0;
    }
    __syncthreads();
    if (tid == 0) {
        const double ts = ordered_sum(S);
        out[(size_t)b * 2] = tg;
        out[(size_t)b * 2 + 1] = ts;
    }
}

}  // namespace fastk
