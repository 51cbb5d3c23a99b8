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
// always current in LDS (64-bit words, or 32-bit when no line sum reaches 2^31) and carries no
// flag bits: the virtual part of a matched cell is recomputed from the embedding's prefix-sum
// intervals when the stage is emitted.  The pass that builds the masks is the inner loop
// (S*S cells per probe, 5 to 6 probes per stage): it reads 32-bit words only - in 64-bit mode
// the low halves, with the few cells of 2^32 and more (virtual bytes piled on the diagonal)
// kept as one more mask per column that is simply OR-ed in, valid while t < 2^32 - and spends
// three VALU instructions per cell: t-1-v with borrow = (v >= t), the running minimum of that
// difference (the largest value under t, from which the next upper bound comes; low halves of
// the large cells may enter it, which can only make that bound less tight), and an
// add-with-carry that shifts the borrow into the mask.  Outputs and status codes as kernel 2.
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
    i64 qmax = 0;      // largest entry of Q: not needed here
    int sh = 0;        // byte counts are in units of 2^sh bytes (0 unless that makes L fit 31 bits)
    const i64 L = embed_into_lds<NR>(wsQ, wsPart, b, S, S, lane, R, PC, EC, diag, PR, ER, qmax, sh);
    if (L <= 0) {
        if (lane == 0) out_num[b] = (int32_t)L;     // -1: invalid input, 0: nothing to send
        return;
    }
    const bool narrow = L < ((i64)1 << 31);
    if (narrow) {
        repack_narrow(R, S * S, lane);
    } else {
        for (int e = lane; e < S * S; e += 64) R[e] &= ~VFLAG;
        wave_sync();
    }

    auto run = [&](auto tag) {
        typedef decltype(tag) V;                // word type of the residuals
        constexpr bool WIDE = sizeof(V) == 8;
        constexpr V VMAX = ~(V)0;               // larger than any residual
        V* Rv = reinterpret_cast<V*>(k9_smem);
        const u32* R32 = reinterpret_cast<const u32*>(k9_smem);
        auto wave_min = [&](V v) -> V {
            if constexpr (sizeof(V) == 4) return wave_min_u32(v);
            else return wave_min_u64(v);
        };
        auto wave_max = [&](V v) -> V {
            if constexpr (sizeof(V) == 4) return wave_max_u32(v);
            else return wave_max_u64(v);
        };
        int row[NR];
        bool valid[NR];
        u32 rowbase[NR];
        int mr[NR];
        u64 ALLC[NR], FREEC[NR];
        u64 cm[NR][NR];
        u64 big[NR][NR];        // 64-bit mode: the cells of the column that hold 2^32 or more
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            row[k] = lane + 64 * k;
            valid[k] = row[k] < S;
            rowbase[k] = valid[k] ? (u32)row[k] * (u32)S : 0u;
            mr[k] = -1;
            const int n = S - 64 * k;
            ALLC[k] = n >= 64 ? ~0ull : (n <= 0 ? 0ull : ((1ull << n) - 1));
#pragma unroll
            for (int w = 0; w < NR; ++w) big[k][w] = 0;
            if constexpr (WIDE) {
                if (valid[k]) {
                    for (int a = 0; a < S; ++a) {
                        const u64 isbig = (Rv[(size_t)a * S + row[k]] >> 32) != 0;
#pragma unroll
                        for (int w = 0; w < NR; ++w)
                            if ((a >> 6) == w) big[k][w] |= isbig << (a & 63);
                    }
                }
            }
        }

        // Column masks of the graph {R >= t}: bit a of cm[k][a / 64] for cell (a, column
        // lane + 64k).  Returns, per lane, an upper bound on the cell values below t seen in its
        // columns that is itself below t (the largest such value, unless a low half of a large
        // cell comes in), 0 if there is none.
        // sfix: 64 * NR when S is exactly that (row strides and loop bounds are then compile-time
        // constants: the loads take immediate offsets and pair up), 0 for any other S
        auto build_s = [&](V t, auto sfix) -> V {
            constexpr int SF = decltype(sfix)::value;
            const int SS = SF ? SF : S;
            if (!WIDE || t <= (V)0xFFFFFFFFu) {
                // 32-bit words (the low halves in 64-bit mode: stride 2)
                constexpr int ST = WIDE ? 2 : 1;
                const u32 tm1 = (u32)t - 1u;
                // smallest t-1-v over the cells with v < t, kept in four independent chains
                u32 dm0 = 0xFFFFFFFFu, dm1 = 0xFFFFFFFFu, dm2 = 0xFFFFFFFFu, dm3 = 0xFFFFFFFFu;
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    const int x = min(row[k], SS - 1);       // lanes past SS re-read the last column
#pragma unroll
                    for (int w = 0; w < NR; ++w) cm[k][w] = 0;
                    for (int a0 = 0; a0 < SS; a0 += 32) {
                        const u32* col = R32 + ((size_t)a0 * SS + x) * ST;
                        u32 m;
                        if (a0 + 32 <= SS) {
                            // Four groups of eight rows, each with its own mask and minimum, so
                            // that no instruction waits for the one before it; rows in descending
                            // order, every step shifting its group's mask left by one.  The borrow
                            // of each subtraction goes through a scalar register pair of its own
                            // (a carry needs two instructions between its producer and consumer).
                            u32 m0 = 0, m1 = 0, m2 = 0, m3 = 0;
                            auto step4 = [&](u32 v0, u32 v1, u32 v2, u32 v3) {
                                u32 d0, d1, d2, d3;
                                u64 c0, c1, c2, c3;
                                asm volatile(
                                    "v_sub_co_u32_e64 %0, %4, %16, %17\n\t"
                                    "v_sub_co_u32_e64 %1, %5, %16, %18\n\t"
                                    "v_sub_co_u32_e64 %2, %6, %16, %19\n\t"
                                    "v_sub_co_u32_e64 %3, %7, %16, %20\n\t"
                                    "v_min_u32_e32 %8, %0, %8\n\t"
                                    "v_min_u32_e32 %9, %1, %9\n\t"
                                    "v_min_u32_e32 %10, %2, %10\n\t"
                                    "v_min_u32_e32 %11, %3, %11\n\t"
                                    "v_addc_co_u32_e64 %12, %4, %12, %12, %4\n\t"
                                    "v_addc_co_u32_e64 %13, %5, %13, %13, %5\n\t"
                                    "v_addc_co_u32_e64 %14, %6, %14, %14, %6\n\t"
                                    "v_addc_co_u32_e64 %15, %7, %15, %15, %7"
                                    : "=&v"(d0), "=&v"(d1), "=&v"(d2), "=&v"(d3),
                                      "=&s"(c0), "=&s"(c1), "=&s"(c2), "=&s"(c3),
                                      "+v"(dm0), "+v"(dm1), "+v"(dm2), "+v"(dm3),
                                      "+v"(m0), "+v"(m1), "+v"(m2), "+v"(m3)
                                    : "v"(tm1), "v"(v0), "v"(v1), "v"(v2), "v"(v3));
                            };
#pragma unroll
                            for (int h = 4; h >= 0; h -= 4) {
                                u32 w16[4][4];
#pragma unroll
                                for (int j = 0; j < 4; ++j)
#pragma unroll
                                    for (int g = 0; g < 4; ++g)
                                        w16[j][g] = col[(size_t)(8 * g + h + j) * SS * ST];
#pragma unroll
                                for (int j = 3; j >= 0; --j)
                                    step4(w16[j][0], w16[j][1], w16[j][2], w16[j][3]);
                            }
                            m = m0 | (m1 << 8) | (m2 << 16) | (m3 << 24);
                        } else {
                            m = 0;
                            for (int i = SS - a0 - 1; i >= 0; --i) {
                                const u32 v = col[(size_t)i * SS * ST];
                                u32 d;
                                asm volatile("v_sub_co_u32_e32 %0, vcc, %3, %4\n\t"
                                             "v_min_u32_e32 %1, %0, %1\n\t"
                                             "s_nop 0\n\t"
                                             "v_addc_co_u32_e32 %2, vcc, %2, %2, vcc"
                                             : "=&v"(d), "+v"(dm0), "+v"(m)
                                             : "v"(tm1), "v"(v)
                                             : "vcc");
                            }
                        }
                        const u64 part = (u64)m << (a0 & 32);
#pragma unroll
                        for (int w = 0; w < NR; ++w)
                            if ((a0 >> 6) == w) cm[k][w] |= part;
                    }
#pragma unroll
                    for (int w = 0; w < NR; ++w) cm[k][w] = valid[k] ? (cm[k][w] | big[k][w]) : 0ull;
                }
                const u32 dmin = min(min(dm0, dm1), min(dm2, dm3));
                return dmin <= tm1 ? (V)(tm1 - dmin) : (V)0;
            } else {
                // thresholds of 2^32 and more: whole 64-bit words
                V below = 0;
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    const int x = min(row[k], SS - 1);
#pragma unroll
                    for (int w = 0; w < NR; ++w) cm[k][w] = 0;
                    for (int a = 0; a < SS; ++a) {
                        const V v = Rv[(size_t)a * SS + x];
                        const bool ge = v >= t;
                        const V u = ge ? (V)0 : v;
                        below = u > below ? u : below;
#pragma unroll
                        for (int w = 0; w < NR; ++w)
                            if ((a >> 6) == w) cm[k][w] |= (u64)ge << (a & 63);
                    }
                    if (!valid[k]) {
#pragma unroll
                        for (int w = 0; w < NR; ++w) cm[k][w] = 0;
                    }
                }
                return below;
            }
        };
        auto build = [&](V t) -> V {
            if (S == 64 * NR) return build_s(t, std::integral_constant<int, 64 * NR>{});
            return build_s(t, std::integral_constant<int, 0>{});
        };

        // FREEC = the columns no row is matched to
        auto free_columns = [&]() {
            wave_sync();
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if (valid[k]) taken[row[k]] = 0;
            wave_sync();
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if (mr[k] >= 0) taken[mr[k]] = 1;
            wave_sync();
#pragma unroll
            for (int k = 0; k < NR; ++k) FREEC[k] = ballot(valid[k] && taken[row[k]] == 0);
        };

        // the residual of each row's matched cell (VMAX for rows without one)
        auto matched_cells = [&](V (&cell)[NR]) {
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                cell[k] = VMAX;
                if (mr[k] >= 0) cell[k] = Rv[rowbase[k] + (u32)mr[k]];
            }
        };

        // Matches rows of U in ascending order, clearing their bits, until one needs the
        // general search: returns that row (-1: U is done).  A row whose own cells
        // reach an unmatched column takes the lowest such column - that is what the canonical
        // search does at its first level - in a loop that works on 32-bit halves of the masks
        // picked at compile time; only the other rows go through the general search, which is
        // instantiated once (match_rows; false as soon as a row cannot be matched).
        auto greedy_rows = [&](u64 (&U)[NR]) -> int {
#pragma unroll
            for (int w = 0; w < NR; ++w) {
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    u32 half[NR];
#pragma unroll
                    for (int k = 0; k < NR; ++k) half[k] = (u32)(cm[k][w] >> (32 * hf));
                    for (u32 z = (u32)(U[w] >> (32 * hf)); z; z &= z - 1) {
                        const int i = __builtin_ctz(z);
                        const int r0 = 64 * w + 32 * hf + i;
                        const u32 bit = 1u << i;
                        u64 N[NR];
#pragma unroll
                        for (int k = 0; k < NR; ++k) N[k] = ballot((half[k] & bit) != 0) & FREEC[k];
                        U[w] &= ~((u64)bit << (32 * hf));
                        if (!mask_any<NR>(N)) return r0;        // needs the general search
                        const int d = mask_lowest<NR>(N);
#pragma unroll
                        for (int k = 0; k < NR; ++k) {
                            mr[k] = row[k] == r0 ? d : mr[k];
                            if ((d >> 6) == k) FREEC[k] &= ~(1ull << (d & 63));
                        }
                    }
                }
            }
            return -1;
        };
        // Paths of two and three hops in straight-line code: r0 -> (column d1 of r0, matched to
        // row a1) -> [(column d2 of a1, matched to row a2) ->] unmatched column d.  They are
        // what the general search finds at its second and third level (lowest unmatched column
        // reached, lowest frontier row as the parent of each column on the way back) and cover
        // nine searches in ten.  False: go deeper.
        auto short_paths = [&](int r0) -> bool {
            auto row_of = [&](int a) -> int {           // mr of a wave-uniform row
                if constexpr (NR == 2) return (a >> 6) ? (int)rdl((u32)mr[1], a & 63) : (int)rdl((u32)mr[0], a & 63);
                else return (int)rdl((u32)mr[0], a);
            };
            auto matched_into = [&](const u64 (&N)[NR], u64 (&F)[NR]) {
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    const int m = mr[k];
                    u64 word;
                    if constexpr (NR == 2) word = m < 64 ? N[0] : N[1];
                    else word = N[0];
                    F[k] = ballot(m >= 0 && ((word >> (m & 63)) & 1));
                }
            };
            auto reached = [&](const u64 (&F)[NR], u64 (&N)[NR]) {
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    u64 cand = 0;
#pragma unroll
                    for (int w = 0; w < NR; ++w) cand |= cm[k][w] & F[w];
                    N[k] = ballot(cand != 0);
                }
            };
            auto parent_in = [&](int d, const u64 (&F)[NR]) -> int {
                u64 par[NR];
                column_mask<NR>(cm, d, par);
#pragma unroll
                for (int w = 0; w < NR; ++w) par[w] &= F[w];
                return mask_lowest<NR>(par);
            };
            u64 F1[NR], N1[NR], F2[NR], N2[NR], fr[NR];
#pragma unroll
            for (int w = 0; w < NR; ++w) F1[w] = (r0 >> 6) == w ? 1ull << (r0 & 63) : 0ull;
            reached(F1, N1);                            // r0's columns, all matched
            matched_into(N1, F2);
            reached(F2, N2);
#pragma unroll
            for (int k = 0; k < NR; ++k) fr[k] = N2[k] & FREEC[k];
            int d, a1, a2 = -1, d2 = -1;
            if (mask_any<NR>(fr)) {
                d = mask_lowest<NR>(fr);
                a1 = parent_in(d, F2);
            } else {
                u64 F3[NR], N3[NR];
#pragma unroll
                for (int k = 0; k < NR; ++k) N2[k] &= ~N1[k];       // newly reached, all matched
                matched_into(N2, F3);
                reached(F3, N3);
#pragma unroll
                for (int k = 0; k < NR; ++k) fr[k] = N3[k] & FREEC[k];
                if (!mask_any<NR>(fr)) return false;
                d = mask_lowest<NR>(fr);
                a2 = parent_in(d, F3);
                d2 = row_of(a2);
                a1 = parent_in(d2, F2);
            }
            const int d1 = row_of(a1);
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                int m = mr[k];
                m = row[k] == r0 ? d1 : m;
                m = row[k] == a1 ? (a2 < 0 ? d : d2) : m;
                m = row[k] == a2 ? d : m;
                mr[k] = m;
                if ((d >> 6) == k) FREEC[k] &= ~(1ull << (d & 63));
            }
            return true;
        };
        auto match_rows = [&](u64 (&U)[NR]) -> bool {
            for (;;) {
                const int r0 = greedy_rows(U);
                if (r0 < 0) return true;
                if (short_paths(r0)) continue;
                if (!bfs_augment<NR>(r0, cm, mr, FREEC, Fh, S, lane)) return false;
            }
        };

        // Does {R >= t} (masks already built) hold a perfect matching?  Starts from what the
        // current matching keeps in that graph, or from nothing (fresh: what it then leaves is
        // the canonical matching of that graph); the matching it leaves lies inside the graph.
        auto feasible = [&](V t, bool fresh) -> bool {
            V cell[NR];
            matched_cells(cell);
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if (fresh || cell[k] < t) mr[k] = -1;
            free_columns();
            u64 U[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) U[k] = ballot(valid[k] && mr[k] < 0);
            return match_rows(U);
        };

        int32_t* srow = out_stages + (size_t)b * max_stages * S;
        i64* brow = out_bytes + (size_t)b * max_stages * S;
        i64* cw = wsC + (size_t)b * max_stages;
        i64 Lrem = L;
        int s = 0, status = 0;
        V hi = (V)L;            // no cell exceeds its line sum
        V gap = 0;              // how far the last bottleneck value lay under its upper bound
        while (Lrem > 0) {
            if (s >= max_stages) { status = -2; break; }
            V lo = 0;           // largest threshold known to admit a perfect matching (0: none yet)
            V t = hi, built = 0;
            const V hi0 = hi;
            V down = 2 * gap;   // while nothing is known to work: step down by this, doubling
            for (;;) {
                const V below = build(t);
                built = t;
                if (feasible(t, false)) {
                    V cell[NR];
                    matched_cells(cell);
                    V m = cell[0];
                    if constexpr (NR == 2) m = cell[1] < m ? cell[1] : m;
                    lo = wave_min(m);               // >= t: the matching also lies in {R >= lo}
                    if (lo >= hi) break;
                } else {
                    hi = wave_max(below);           // thresholds in (hi, t] give the graph of t again
                    if (hi <= lo) break;
                }
                if (lo == 0 && down != 0 && hi > down) {
                    t = hi - down;                  // consecutive bottleneck values lie close together
                    down *= 2;
                } else {
                    t = lo + (hi - lo + 1) / 2;     // lo < t <= hi
                }
            }
            if (lo == 0) { status = -3; break; }    // not even the support holds a perfect matching
            const V tstar = lo;
            if (hi0 > tstar) gap = hi0 - tstar;

            // the stage's matching: from nothing, whatever the probes left behind
            if (built != tstar) (void)build(tstar);
            if (!feasible(tstar, true)) { status = -3; break; }

            V cell[NR];
            matched_cells(cell);
            V m = cell[0];
            if constexpr (NR == 2) m = cell[1] < m ? cell[1] : m;
            const V c = wave_min(m);
            if (c != tstar) { status = -3; break; }
            u64 crossed[NR];    // rows whose cell just fell under 2^32
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                bool cross = false;
                if (valid[k]) {
                    const int d = mr[k];
                    const V v = cell[k];
                    // virtual bytes the embedding put in the cell
                    const i64 l = max(PR[k], PC[d]);
                    const i64 h = min(ER[k], EC[d]);
                    const i64 av = (h > l ? h - l : 0) + (d == row[k] ? diag[k] : 0);
                    const i64 real_left = (i64)v > av ? (i64)v - av : 0;
                    const i64 real = min((i64)c, real_left);
                    srow[row[k]] = real > 0 ? d : -1;
                    brow[row[k]] = real << sh;
                    const V left = v - c;
                    Rv[rowbase[k] + (u32)d] = left;
                    if constexpr (WIDE) cross = (v >> 32) != 0 && (left >> 32) == 0;
                }
                crossed[k] = ballot(cross);
            }
            if constexpr (WIDE) {
#pragma unroll
                for (int kr = 0; kr < NR; ++kr)
                    for (u64 z = crossed[kr]; z; z &= z - 1) {
                        const int al = __builtin_ctzll(z);          // row 64 * kr + al
                        const int d = (int)rdl((u32)mr[kr], al);
#pragma unroll
                        for (int k = 0; k < NR; ++k)
                            if ((d >> 6) == k && lane == (d & 63)) big[k][kr] &= ~(1ull << al);
                    }
            }
            if (lane == 0) cw[s] = (i64)c << sh;
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
