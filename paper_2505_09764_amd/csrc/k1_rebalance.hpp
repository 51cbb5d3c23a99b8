// Kernel 1: server aggregation, sender balancing and collapse.
//
// One workgroup per (matrix b, source server a) handles the G x N row block of
// the traffic matrix that belongs to server a:
//   phase A  reads the block once and reduces every cross-server tile row to its
//            row sum r_i(a,d) (paper Section 4.1 "Example setup": a tile's row
//            sums are what each GPU sends to that server);
//   phase B  per tile: tile total T[a][d], lane targets floor/ceil(T/G), each
//            row's surplus or deficit and its position (prefix sum) among the
//            tile's surpluses / deficits (Section 4.1 "Mitigating sender skew");
//            the per-lane server entry Q[a][d] = ceil(T/G) of the merged peer
//            transfer (Section 4.1 "Mitigating receiver skew", Section 4.2 Fig. 6);
//   phase C  writes the lane-routing matrix X.  Pouring surpluses into deficits in
//            ascending index order means surplus row i covers the byte interval
//            [PS_i, PS_i + s_i) and deficit row k the interval [PD_k, PD_k + d_k)
//            of the same line, so X[i][k] is the length of their intersection -
//            every output element is independent of the others.
// The block also leaves, for the cost model, the largest per-GPU hand-off
// volume (balancing) and intra-server volume of its server.
//
// HBM traffic: the row block is read once (8*G*N bytes) and X written once
// (8*G*N bytes); everything else lives in LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fastk {

typedef long long i64;
typedef unsigned long long u64;

struct alignas(16) i64x2 { i64 x, y; };

constexpr int K1_THREADS = 256;
constexpr u64 K1_SURPLUS_BIT = 1ull << 63;

// Per-block record left for kernels 2 and 3: [b][a][4]
//   0: max over the server's GPUs of max(bytes handed off, bytes handed in)
//   1: max over the server's GPUs of max(intra-server bytes out, in)
//   2: 1 if a negative off-diagonal entry was seen in the block
//   3: sum_d T[a][d]
constexpr int K1_PART = 4;

inline size_t k1_lds_bytes(int S, int G) {
    return (size_t)S * G * 4 * sizeof(i64) + (size_t)(4 * G + 2) * sizeof(i64);
}

template <int G, bool VEC>
__global__ void __launch_bounds__(K1_THREADS)
k1_rebalance(const i64* __restrict__ traffic, i64* __restrict__ X, i64* __restrict__ wsT,
             i64* __restrict__ wsQ, i64* __restrict__ wsPart, int S) {
    extern __shared__ __align__(16) unsigned char k1_smem[];
    const int a = blockIdx.x;
    const int b = blockIdx.y;
    const int N = S * G;
    const int P = S * G;                 // tile rows in the block, index p = d*G + i
    i64* r = reinterpret_cast<i64*>(k1_smem);
    u64* lo = reinterpret_cast<u64*>(r + P);
    i64* hi = reinterpret_cast<i64*>(lo + P);
    i64* kept = hi + P;
    i64* acc_out = kept + P;             // [G] bytes handed off per GPU
    i64* acc_in = acc_out + G;           // [G] bytes handed in per GPU
    i64* intra_in = acc_in + G;          // [G] intra-server bytes received per GPU
    i64* intra_out = intra_in + G;       // [G]
    i64* misc = intra_out + G;           // [0] negative flag, [1] sum_d T[a][d]
    const int tid = threadIdx.x;

    if (tid < 4 * G + 2) acc_out[tid] = 0;
    __syncthreads();

    const i64* blk = traffic + ((size_t)b * N + (size_t)a * G) * N;

    // ---- phase A: tile row sums.  Tile rows are taken in (i, d) order so that
    // consecutive threads read consecutive tiles of one GPU row.
    bool neg = false;
    for (int t = tid; t < P; t += K1_THREADS) {
        const int i = t / S;
        const int d = t - i * S;
        const i64* src = blk + (size_t)i * N + (size_t)d * G;
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
        i64 sum = 0;
        if (d == a) {
#pragma unroll
            for (int j = 0; j < G; ++j) {
                if (j != i) {                       // the GPU diagonal uses no link
                    neg |= v[j] < 0;
                    sum += v[j];
                    atomicAdd(reinterpret_cast<u64*>(&intra_in[j]), (u64)v[j]);
                }
            }
            intra_out[i] = sum;
        } else {
#pragma unroll
            for (int j = 0; j < G; ++j) {
                neg |= v[j] < 0;
                sum += v[j];
            }
        }
        r[d * G + i] = sum;
    }
    if (neg) misc[0] = 1;
    __syncthreads();

    // ---- phase B: one thread per tile row (d, i)
    for (int p = tid; p < P; p += K1_THREADS) {
        const int d = p / G;
        const int i = p - d * G;
        if (d == a) {
            lo[p] = 0;
            hi[p] = 0;
            kept[p] = 0;
            if (i == 0) {
                wsT[((size_t)b * S + a) * S + d] = 0;
                wsQ[((size_t)b * S + a) * S + d] = 0;
            }
            continue;
        }
        i64 rr[G];
        i64 tot = 0;
#pragma unroll
        for (int k = 0; k < G; ++k) {
            rr[k] = r[d * G + k];
            tot += rr[k];
        }
        const i64 q = tot / G;
        const int rho = (int)(tot - q * G);
        i64 ps = 0, pd = 0, my_s = 0, my_d = 0, my_t = 0;
#pragma unroll
        for (int k = 0; k < G; ++k) {
            const i64 tk = q + (k < rho ? 1 : 0);
            const i64 sk = rr[k] > tk ? rr[k] - tk : 0;
            const i64 dk = tk > rr[k] ? tk - rr[k] : 0;
            if (k < i) { ps += sk; pd += dk; }
            if (k == i) { my_s = sk; my_d = dk; my_t = tk; }
        }
        if (my_s > 0) {
            lo[p] = (u64)ps | K1_SURPLUS_BIT;
            hi[p] = ps + my_s;
            atomicAdd(reinterpret_cast<u64*>(&acc_out[i]), (u64)my_s);
        } else {
            lo[p] = (u64)pd;
            hi[p] = pd + my_d;
            if (my_d > 0) atomicAdd(reinterpret_cast<u64*>(&acc_in[i]), (u64)my_d);
        }
        kept[p] = rr[i] < my_t ? rr[i] : my_t;
        if (i == 0) {
            wsT[((size_t)b * S + a) * S + d] = tot;
            wsQ[((size_t)b * S + a) * S + d] = q + (rho > 0 ? 1 : 0);
            atomicAdd(reinterpret_cast<u64*>(&misc[1]), (u64)tot);
        }
    }
    __syncthreads();

    if (tid == 0) {
        i64 bal = 0, intra = 0;
        for (int i = 0; i < G; ++i) {
            bal = max(bal, max(acc_out[i], acc_in[i]));
            intra = max(intra, max(intra_out[i], intra_in[i]));
        }
        i64* part = wsPart + ((size_t)b * S + a) * K1_PART;
        part[0] = bal;
        part[1] = intra;
        part[2] = misc[0];
        part[3] = misc[1];
    }

    // ---- phase C: lane-routing matrix, coalesced along each GPU row
    i64* xblk = X + ((size_t)b * N + (size_t)a * G) * N;
    auto cell = [&](int d, int i, int k, u64 lo_i, i64 hi_i, i64 kept_i) -> i64 {
        if (d == a) return 0;
        if (k == i) return kept_i;
        if (!(lo_i & K1_SURPLUS_BIT)) return 0;      // a deficit row hands nothing off
        const u64 lo_k = lo[d * G + k];
        if (lo_k & K1_SURPLUS_BIT) return 0;         // a surplus row takes nothing in
        const i64 l = max((i64)(lo_i & ~K1_SURPLUS_BIT), (i64)lo_k);
        const i64 h = min(hi_i, hi[d * G + k]);
        return h > l ? h - l : 0;
    };
    if constexpr (VEC) {
        const int half = N / 2;
        for (int e = tid; e < G * half; e += K1_THREADS) {
            const int i = e / half;
            const int h = (e - i * half) * 2;
            const int d = h / G;
            const int k = h - d * G;
            const int p = d * G + i;
            const u64 lo_i = lo[p];
            const i64 hi_i = hi[p];
            const i64 kept_i = kept[p];
            i64x2 w;
            w.x = cell(d, i, k, lo_i, hi_i, kept_i);
            w.y = cell(d, i, k + 1, lo_i, hi_i, kept_i);
            *reinterpret_cast<i64x2*>(xblk + (size_t)i * N + h) = w;
        }
    } else {
        for (int e = tid; e < G * N; e += K1_THREADS) {
            const int i = e / N;
            const int h = e - i * N;
            const int d = h / G;
            const int k = h - d * G;
            const int p = d * G + i;
            xblk[(size_t)i * N + h] = cell(d, i, k, lo[p], hi[p], kept[p]);
        }
    }
}

}  // namespace fastk
