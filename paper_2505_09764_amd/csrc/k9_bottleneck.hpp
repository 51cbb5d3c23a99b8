// Kernel 9: decomposition into fewer, larger stages.
//
// The paper notes (Section 4.4 "Number of stages") that fewer stages are preferable - each one
// costs a synchronisation - and that the minimum is NP-hard, and settles for any valid
// decomposition.  This kernel is a greedy variant that is not in the paper: every stage takes
// a bottleneck assignment of the residual R = Q + A, i.e. a perfect matching whose smallest
// cell is as large as possible, so each stage removes the most weight one stage can.  On the
// skewed MoE matrices of the benchmark this gives about 14 times fewer stages at 128 servers
// (4 times at 32), for a synthesis that is several times slower than kernel 2.
//
// Per stage:
//   1. the bottleneck value t* = the largest t for which the cells holding at least t contain
//      a perfect matching.  t* is a cell value and never exceeds the previous stage's weight
//      (the residual only shrinks), so the search runs between lo (a threshold known to work)
//      and hi (an upper bound): probe t - first hi itself, which succeeds for about a quarter
//      of the stages, then the midpoint -, build the column masks of the graph {R >= t} by one
//      pass over LDS, keep of the current matching what lies in that graph and augment the
//      rows that lost their cell.  Success raises lo to the smallest cell of the matching
//      found; failure lowers hi to the largest cell value below t (collected during the same
//      pass), which skips every threshold that would give the same graph again.  The partial
//      matching left by a failed probe stays valid for every lower threshold.
//   2. the stage's matching = the canonical matching of {R >= t*}, built from nothing by
//      augmenting rows 0..S-1 in order (same search as kernel 2; a row whose own cells reach
//      an unmatched column takes the lowest such column without entering the general search).
//      Building it afresh makes the result a function of the residual alone, however the
//      search for t* went.
//   3. weight c = t*; real bytes of a cell are consumed before virtual ones; rows whose cell
//      has no real bytes left are idle (-1); the matched cells lose c in LDS.
//
// One wavefront per matrix; lane l owns rows and columns l, l + 64.  The residual matrix is
// always current in LDS (64-bit words, or 32-bit when no line sum reaches 2^31); the virtual
// part of a cell is recomputed from the embedding's prefix-sum intervals when the cell is
// flagged.  Outputs and status codes as kernel 2.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <limits>
#include <type_traits>

#include "matching.hpp"

namespace fastk {

constexpr int K9_THREADS = 64;

// R[S][S], column deficit intervals PC[S], EC[S], frontier history [(S+2)][2], one int32 per
// column (which columns are matched)
__host__ __device__ inline size_t k9_lds_bytes(int S) {
    return (size_t)S * S * 8 + (size_t)2 * S * 8 + (size_t)(S + 2) * 16 + (((size_t)S * 4 + 15) & ~(size_t)15);
}

template <int NR>
__global__ void __launch_bounds__(K9_THREADS)
k9_bottleneck(const i64* __restrict__ wsQ, const i64* __restrict__ wsPart,
              int32_t* __restrict__ out_stages, i64* __restrict__ out_bytes,
              int32_t* __restrict__ out_num, i64* __restrict__ wsC, int S, int max_stages) {
    extern __shared__ __align__(16) unsigned char k9_smem[];
    u64* R = reinterpret_cast<u64*>(k9_smem);
    i64* PC = reinterpret_cast<i64*>(R + (size_t)S * S);
    i64* EC = PC + S;
    u64* Fh = reinterpret_cast<u64*>(EC + S);       // [level][2]
    int32_t* taken = reinterpret_cast<int32_t*>(Fh + (size_t)(S + 2) * 2);
    const int b = blockIdx.x;
    const int lane = threadIdx.x;

    i64 diag[NR], PR[NR], ER[NR];
    const i64 L = embed_into_lds<NR>(wsQ, wsPart, b, S, lane, R, PC, EC, diag, PR, ER);
    if (L <= 0) {
        if (lane == 0) out_num[b] = (int32_t)L;     // -1: invalid input, 0: nothing to send
        return;
    }
    const bool narrow = L < ((i64)1 << 31);
    if (narrow) repack_narrow(R, S, lane);

    auto run = [&](auto tag) {
        typedef decltype(tag) V;                // word type of the residuals
        constexpr V VF = (V)((V)1 << (sizeof(V) * 8 - 1));   // the cell holds virtual bytes
        constexpr V VMAX = (V)~VF;                            // larger than any residual
        V* Rv = reinterpret_cast<V*>(k9_smem);
        auto wave_min = [&](V v) -> V {
            if constexpr (sizeof(V) == 4) return wave_min_u32(v);
            else return wave_min_u64(v);
        };
        auto wave_max = [&](V v) -> V {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const V o = __shfl_xor(v, off, 64);
                v = o > v ? o : v;
            }
            return v;
        };
        int row[NR];
        bool valid[NR];
        u32 rowbase[NR];
        int mr[NR];
        u64 ALLC[NR], FREEC[NR];
        u64 cm[NR][NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            row[k] = lane + 64 * k;
            valid[k] = row[k] < S;
            rowbase[k] = valid[k] ? (u32)row[k] * (u32)S : 0u;
            mr[k] = -1;
            const int n = S - 64 * k;
            ALLC[k] = n >= 64 ? ~0ull : (n <= 0 ? 0ull : ((1ull << n) - 1));
        }

        // Column masks of the graph {R >= t}: bit a of cm[k][a / 64] for cell (a, column
        // lane + 64k).  Returns, per lane, the largest cell value below t seen in its columns.
        auto build = [&](V t) -> V {
            V below = 0;
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const int x = min(row[k], S - 1);       // lanes past S re-read the last column
#pragma unroll
                for (int w = 0; w < NR; ++w) cm[k][w] = 0;
                for (int a0 = 0; a0 < S; a0 += 32) {
                    const int n = min(32, S - a0);
                    u32 m = 0;
                    const V* col = Rv + (size_t)a0 * S + x;
#pragma unroll 8
                    for (int i = 0; i < n; ++i) {
                        const V v = col[(size_t)i * S] & (V)~VF;
                        const bool ge = v >= t;
                        m |= (u32)ge << i;
                        const V u = ge ? (V)0 : v;
                        below = u > below ? u : below;
                    }
                    const u64 part = (u64)m << (a0 & 32);
#pragma unroll
                    for (int w = 0; w < NR; ++w)
                        if ((a0 >> 6) == w) cm[k][w] |= part;
                }
                if (!valid[k]) {
#pragma unroll
                    for (int w = 0; w < NR; ++w) cm[k][w] = 0;
                }
            }
            return below;
        };

        // FREEC = the columns no row is matched to
        auto free_columns = [&]() {
            __syncthreads();
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if (valid[k]) taken[row[k]] = 0;
            __syncthreads();
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if (mr[k] >= 0) taken[mr[k]] = 1;
            __syncthreads();
#pragma unroll
            for (int k = 0; k < NR; ++k) FREEC[k] = ballot(valid[k] && taken[row[k]] == 0);
        };

        // the residual of each row's matched cell, flag included (VMAX for rows without one)
        auto matched_cells = [&](V (&cell)[NR]) {
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                cell[k] = VMAX;
                if (mr[k] >= 0) cell[k] = Rv[rowbase[k] + (u32)mr[k]];
            }
        };

        auto augment = [&](int r0) -> bool {
            // level 1 by hand: the lowest unmatched column among r0's own cells
            u64 N[NR];
            const u64 bit = 1ull << (r0 & 63);
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                u64 word;
                if constexpr (NR == 2) word = (r0 >> 6) ? cm[k][1] : cm[k][0];
                else word = cm[k][0];
                N[k] = ballot((word & bit) != 0) & FREEC[k];
            }
            if (mask_any<NR>(N)) {
                const int d = mask_lowest<NR>(N);
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    mr[k] = row[k] == r0 ? d : mr[k];
                    if ((d >> 6) == k) FREEC[k] &= ~(1ull << (d & 63));
                }
                return true;
            }
            return bfs_augment<NR>(r0, cm, mr, FREEC, Fh, S, lane);
        };

        // Does {R >= t} (masks already built) hold a perfect matching?  Starts from what the
        // current matching keeps in that graph; the matching it leaves lies inside the graph.
        auto feasible = [&](V t) -> bool {
            V cell[NR];
            matched_cells(cell);
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if ((cell[k] & (V)~VF) < t) mr[k] = -1;
            free_columns();
            u64 U[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) U[k] = ballot(valid[k] && mr[k] < 0);
#pragma unroll
            for (int w = 0; w < NR; ++w)
                for (u64 z = U[w]; z; z &= z - 1)
                    if (!augment(64 * w + __builtin_ctzll(z))) return false;
            return true;
        };

        int32_t* srow = out_stages + (size_t)b * max_stages * S;
        i64* brow = out_bytes + (size_t)b * max_stages * S;
        i64* cw = wsC + (size_t)b * max_stages;
        i64 Lrem = L;
        int s = 0, status = 0;
        V hi = (V)L;            // no cell exceeds its line sum
        while (Lrem > 0) {
            if (s >= max_stages) { status = -2; break; }
            V lo = 0;           // largest threshold known to admit a perfect matching (0: none yet)
            V t = hi, built = 0;
            for (;;) {
                const V below = build(t);
                built = t;
                if (feasible(t)) {
                    V cell[NR];
                    matched_cells(cell);
                    V m = cell[0] & (V)~VF;
                    if constexpr (NR == 2) {
                        const V m1 = cell[1] & (V)~VF;
                        m = m1 < m ? m1 : m;
                    }
                    lo = wave_min(m);               // >= t: the matching also lies in {R >= lo}
                    if (lo >= hi) break;
                } else {
                    hi = wave_max(below);           // thresholds in (hi, t] give the graph of t again
                    if (hi <= lo) break;
                }
                t = lo + (hi - lo + 1) / 2;         // lo < t <= hi
            }
            if (lo == 0) { status = -3; break; }    // not even the support holds a perfect matching
            const V tstar = lo;

            if (built != tstar) (void)build(tstar);
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                mr[k] = -1;
                FREEC[k] = ALLC[k];
            }
            bool ok = true;
            for (int r0 = 0; r0 < S && ok; ++r0) ok = augment(r0);
            if (!ok) { status = -3; break; }

            V cell[NR];
            matched_cells(cell);
            V m = cell[0] & (V)~VF;
            if constexpr (NR == 2) {
                const V m1 = cell[1] & (V)~VF;
                m = m1 < m ? m1 : m;
            }
            const V c = wave_min(m);
            if (c != tstar) { status = -3; break; }
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                if (valid[k]) {
                    const int d = mr[k];
                    const V v = cell[k] & (V)~VF;
                    i64 av = 0;                      // virtual bytes the embedding put in the cell
                    if (cell[k] & VF) {
                        const i64 l = max(PR[k], PC[d]);
                        const i64 h = min(ER[k], EC[d]);
                        av = (h > l ? h - l : 0) + (d == row[k] ? diag[k] : 0);
                    }
                    const i64 real_left = (i64)v > av ? (i64)v - av : 0;
                    const i64 real = min((i64)c, real_left);
                    srow[row[k]] = real > 0 ? d : -1;
                    brow[row[k]] = real;
                    Rv[rowbase[k] + (u32)d] = (V)(v - c) | (cell[k] & VF);
                }
            }
            if (lane == 0) cw[s] = (i64)c;
            ++s;
            srow += S;
            brow += S;
            Lrem -= (i64)c;
            hi = c;             // the next bottleneck value cannot be larger
        }
        if (lane == 0) out_num[b] = status < 0 ? status : s;
    };
    if (narrow) run((u32)0);
    else run((u64)0);
}

}  // namespace fastk
