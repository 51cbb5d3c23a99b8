// Kernel 2: embedding and Birkhoff decomposition of the server-level matrix.
//
// One wavefront (64 lanes) per traffic matrix.  The stage loop of Birkhoff's
// decomposition (paper Section 4.4 "Birkhoff's decomposition: overview") is a
// chain of dependent steps - find a perfect matching, take the smallest matched
// entry as the stage weight, subtract, repair the matching - and a generic
// matrix needs about (S-1)^2 stages, so the design goal is the fewest
// instructions on the dependent path of one stage, not memory throughput (one
// wavefront issues an instruction every 5 to 8 cycles whatever its kind):
//   * a single wavefront owns the matrix, so no step needs a workgroup barrier;
//     lane l owns rows l, l+64 and columns l, l+64 (S <= 128);
//   * the residual matrix R = Q + A lives in LDS (S*S int64) and is only touched
//     when the matching changes: the residual of each row's matched cell is held
//     in a register and written back when the row is re-matched;
//   * the support of R is kept as one S-bit row mask per column in registers;
//     frontiers, visited sets and the set of unmatched columns are wave-uniform
//     bit masks, so one breadth-first level is a few AND/compare operations per
//     lane plus ballots, and "does the frontier reach an unmatched column" is a
//     scalar test on that column's mask;
//   * parents are not stored: the parent of a column is recomputed while the
//     augmenting path is flipped, as the lowest set bit of (its support mask AND
//     the frontier of the level that reached it);
//   * almost every stage exhausts exactly one cell (r0, f) and is repaired by a
//     path of at most three levels; that case runs as straight-line code, every
//     other case goes through the general search;
//   * the virtual matrix A of the embedding (Section 4.4 "Adapting an arbitrary
//     matrix to a valid form") is never stored: pouring row deficits into column
//     deficits in ascending order makes A[a][d] the overlap of two prefix-sum
//     intervals (plus the diagonal term); cells that hold virtual bytes are
//     flagged in the top bit of their LDS word and the overlap is recomputed only
//     when such a cell gets matched;
//   * no residual exceeds L, the largest row/column sum, so when L < 2^31 the matrix
//     is repacked in place to 32-bit words and the stage loop runs on 32-bit
//     registers; when S fills the lane slots exactly (64 or 128) the stage loop
//     carries no bounds predicates.  Predicated LDS writes and mid-loop exits cost a
//     lone wavefront far more than their instruction count suggests (exec-mask
//     save/restore pairs, scalar branches at 11-13 cycles per instruction), so the
//     dependent path avoids them: unconditional write-back of the old matched cell,
//     the stage weight stored by every lane, error exits checked once per stage.
//
// Canonical choices that make the result a function of the matrix alone (the
// paper leaves them open): level-synchronous search from one unmatched row, the
// lowest-numbered frontier row becomes the parent of a newly reached column, the
// search stops at the first level that reaches an unmatched column and takes the
// lowest-numbered one; first matching = rows 0..S-1 augmented in order; stage
// weight = smallest matched residual; real bytes of a cell are consumed before
// virtual ones; after a stage only rows whose matched cell reached zero are
// unmatched (all first), then re-augmented in ascending order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <limits>
#include <type_traits>

#include "k3_cost.hpp"
#include "matching.hpp"

namespace fastk {

constexpr int K2_THREADS = 64;

// R[S][S], column deficit intervals PC[S], EC[S], frontier history [(S+2)][2]
__host__ __device__ inline size_t k2_lds_data_bytes(int S) {
    return (size_t)S * S * 8 + (size_t)2 * S * 8 + (size_t)(S + 2) * 16;
}
// ... plus one spare word per lane slot and one in front: the lane slots that hold no row
// (S below 64 * NR) read and write there, so the per-stage reload needs no bounds predicate
inline size_t k2_lds_bytes(int S) { return k2_lds_data_bytes(S) + (size_t)(2 * 64 + 1) * 8; }

// NR = rows (and columns) per lane: 1 for S <= 64, 2 for S <= 128.
// NR: rows and columns per lane; FULL: S == 64 * NR, every lane slot holds a real row (the
// stage rows are then stored without a per-lane bounds predicate).
template <int NR, bool FULL>
__device__ __forceinline__ void
k2_matrix(const i64* __restrict__ wsQ, const i64* __restrict__ wsPart,
          int32_t* __restrict__ out_stages, i64* __restrict__ out_bytes,
          int32_t* __restrict__ out_num, i64* __restrict__ wsC, int S_arg, int max_stages,
          int b, int lane, unsigned char* k2_smem) {
    const int S = FULL ? 64 * NR : S_arg;       // FULL: a compile-time constant
    u64* R = reinterpret_cast<u64*>(k2_smem);
    i64* PC = reinterpret_cast<i64*>(R + (size_t)S * S);
    i64* EC = PC + S;
    u64* Fh = reinterpret_cast<u64*>(EC + S);       // [level][2]

    i64 diag[NR], PR[NR], ER[NR];
    const i64 L = embed_into_lds<NR>(wsQ, wsPart, b, S, lane, R, PC, EC, diag, PR, ER);
    if (L <= 0) {
        if (lane == 0) out_num[b] = (int32_t)L;     // -1: invalid input, 0: nothing to send
        return;
    }

    // support masks: bit a of cm[k][a/64] set while R[a][column lane+64k] > 0
    u64 cm[NR][NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int x = lane + 64 * k;
#pragma unroll
        for (int w = 0; w < NR; ++w) cm[k][w] = 0;
        if (x < S) {
            for (int a = 0; a < S; ++a) {
                const u64 pos = (R[(size_t)a * S + x] & ~VFLAG) != 0;
#pragma unroll
                for (int w = 0; w < NR; ++w)
                    if ((a >> 6) == w) cm[k][w] |= pos << (a & 63);
            }
        }
    }

    // Residuals never exceed L, so when L < 2^31 the whole stage loop runs on 32-bit words: the
    // residual matrix is repacked in place (flag in bit 31) and every per-stage subtraction,
    // comparison and select is one instruction instead of two.
    const bool narrow = L < ((i64)1 << 31);
    if (narrow) repack_narrow(R, S, lane);
    auto run = [&](auto tag) {
        typedef decltype(tag) V;                // word type of the residuals
        typedef std::make_signed_t<V> SV;
        constexpr V VF = (V)((V)1 << (sizeof(V) * 8 - 1));   // the cell holds virtual bytes
        V* Rv = reinterpret_cast<V*>(k2_smem);
        auto wave_min = [&](V v) -> V {
            if constexpr (sizeof(V) == 4) return wave_min_u32(v);
            else return wave_min_u64(v);
        };
        int lid[NR];
        u32 rowbase[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            lid[k] = lane + 64 * k;
            // a slot without a row keeps mr = loaded = -1: base + (-1) is its spare word
            // (the first reload, before any row is loaded, reads base + 0: the next spare word)
            const u32 spare = (u32)(k2_lds_data_bytes(S) / sizeof(V)) + (u32)(lane + 64 * k) + 1u;
            rowbase[k] = lane + 64 * k < S ? (u32)(lane + 64 * k) * (u32)S : spare;
        }
        int mr[NR], loaded[NR];
        SV rv[NR], rl[NR];
        V vfl[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            mr[k] = -1;
            loaded[k] = -1;
            rv[k] = 0;
            rl[k] = 0;
            vfl[k] = 0;
        }
        u64 FREEC[NR];     // unmatched columns (wave-uniform)
#pragma unroll
        for (int w = 0; w < NR; ++w) {
            const int n = S - 64 * w;
            FREEC[w] = n >= 64 ? ~0ull : (n <= 0 ? 0ull : ((1ull << n) - 1));
        }

        // cm of column d (uniform) as uniform words
        auto col_mask = [&](int d, u64 (&out)[NR]) {
            const int dl = d & 63;
#pragma unroll
            for (int w = 0; w < NR; ++w) {
                if constexpr (NR == 2) out[w] = (d >> 6) ? rdl64(cm[1][w], dl) : rdl64(cm[0][w], dl);
                else out[w] = rdl64(cm[0][w], dl);
            }
        };
        auto lowest = [&](const u64 (&m)[NR]) -> int {
            if constexpr (NR == 2) return m[0] ? __builtin_ctzll(m[0]) : 64 + __builtin_ctzll(m[1]);
            else return __builtin_ctzll(m[0]);
        };
        auto any = [&](const u64 (&m)[NR]) -> bool {
            if constexpr (NR == 2) return (m[0] | m[1]) != 0;
            else return m[0] != 0;
        };

        auto augment = [&](int r0) -> bool {
            return bfs_augment<NR>(r0, cm, mr, FREEC, Fh, S, lane);
        };

        // Make rv / rl describe the cell each row is matched to now.  Loads are
        // issued for every row (cheap, no exec juggling) and kept only where the
        // match changed; the old cell's residual is written back where it is non-zero.
        // FIRST: the call after the initial matching, when nothing has been loaded yet.  Later
        // calls (every row matched; lane slots without a row work on their spare word) write the
        // old cell back unconditionally - for an unchanged row that rewrites what LDS already
        // holds, for an exhausted cell it stores the zero that is its true residual - which saves
        // the predicates and the exec juggling on the dependent path.
        auto sync_matched = [&](auto first_tag) {
            constexpr bool FIRST = decltype(first_tag)::value;
            constexpr bool PLAIN = !FIRST;
            V x[NR];
            bool ch[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                ch[k] = mr[k] != loaded[k];
                if constexpr (PLAIN) {
                    Rv[rowbase[k] + (u32)loaded[k]] = (V)rv[k] | vfl[k];
                    x[k] = Rv[rowbase[k] + (u32)mr[k]];
                } else {
                    if (ch[k] && rv[k] > 0) Rv[rowbase[k] + (u32)loaded[k]] = (V)rv[k] | vfl[k];
                    x[k] = Rv[rowbase[k] + (u32)max(mr[k], 0)];
                }
            }
            u64 anyv = 0;
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const V val = x[k] & (V)~VF;
                const V fl = x[k] & VF;
                rv[k] = ch[k] ? (SV)val : rv[k];
                rl[k] = ch[k] ? (SV)val : rl[k];
                anyv |= ballot(ch[k]) & ballot(fl != 0);
                vfl[k] = ch[k] ? fl : vfl[k];
                loaded[k] = mr[k];
            }
            if (__builtin_expect(anyv != 0, 0)) {
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    if (ch[k] && vfl[k] != 0) {
                        const int d = mr[k];
                        const i64 l = max(PR[k], PC[d]);
                        const i64 h = min(ER[k], EC[d]);
                        const i64 av = (h > l ? h - l : 0) + (d == lid[k] ? diag[k] : 0);
                        rl[k] = (i64)rv[k] > av ? (SV)((i64)rv[k] - av) : (SV)0;
                    }
                }
            }
        };

        int status = 0;
        for (int r0 = 0; r0 < S; ++r0)
            if (!augment(r0)) { status = -3; break; }
        if (status < 0) {
            if (lane == 0) out_num[b] = status;
            return;
        }
        sync_matched(std::true_type{});
#pragma unroll
        for (int k = 0; k < NR; ++k)
            if (lane + 64 * k >= S) rv[k] = std::numeric_limits<SV>::max();     // never the minimum, never zero

        int32_t* stg = out_stages + (size_t)b * max_stages * S;
        i64* byt = out_bytes + (size_t)b * max_stages * S;
        i64* cw = wsC + (size_t)b * max_stages;
        i64 Lrem = L;
        int s = 0;
        int32_t* srow = stg;
        i64* brow = byt;
        // mr of a uniform row
        auto mr_of = [&](int a) -> int {
            if constexpr (NR == 2) {
                const int x0 = (int)rdl((u32)mr[0], a & 63), x1 = (int)rdl((u32)mr[1], a & 63);
                return (a & 64) ? x1 : x0;
            } else {
                return (int)rdl((u32)mr[0], a);
            }
        };
        auto set_mr = [&](int a, int d) {
#pragma unroll
            for (int k = 0; k < NR; ++k) mr[k] = lid[k] == a ? d : mr[k];
        };
        // columns (as a uniform mask per column slot) adjacent to any row of F
        auto expand = [&](const u64 (&F)[NR], u64 (&N)[NR]) {
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                u64 cand = 0;
#pragma unroll
                for (int w = 0; w < NR; ++w) cand |= cm[k][w] & F[w];
                N[k] = ballot(cand != 0);
            }
        };
        // rows (uniform mask per row slot) whose matched column is in N
        auto rows_matched_into = [&](const u64 (&N)[NR], u64 (&F)[NR]) {
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const int m = mr[k];
                u64 word;
                if constexpr (NR == 2) word = m < 64 ? N[0] : N[1];
                else word = N[0];
                F[k] = ballot(m >= 0 && ((word >> (m & 63)) & 1));
            }
        };

        for (;;) {
            if (__builtin_expect(s >= max_stages, 0)) { status = -2; break; }
            V mine = (V)rv[0];
            if constexpr (NR == 2) mine = (V)rv[1] < mine ? (V)rv[1] : mine;
            const i64 c64 = (i64)wave_min(mine);    // stage weight: wave-uniform, fits SV
            const SV c = (SV)c64;
            u64 Z[NR];
            bool zero[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const SV real = c < rl[k] ? c : rl[k];
                rl[k] -= real;
                rv[k] -= c;
                if (FULL || lid[k] < S) {
                    srow[lid[k]] = real > 0 ? mr[k] : -1;
                    brow[lid[k]] = (i64)real;
                }
                zero[k] = rv[k] == 0;
                Z[k] = ballot(zero[k]);
            }
            cw[s] = c64;      // every lane stores the same word: no divergent branch on the path
            ++s;
            srow += S;
            brow += S;
            Lrem -= c64;
            if (__builtin_expect(Lrem == 0, 0)) break;

            int nz = 0;
#pragma unroll
            for (int w = 0; w < NR; ++w) nz += __builtin_popcountll(Z[w]);
            if (__builtin_expect(nz == 1, 1)) {
                // ---- fast path: one exhausted cell (r0, f); f is the only unmatched column.
                // Row r0 keeps naming f as its column until the flip; f is not adjacent to
                // r0 any more, so r0 cannot enter a frontier through it.
                const int r0 = lowest(Z);
                const int f = mr_of(r0);
                const u64 bit0 = 1ull << (r0 & 63);
                u64 cmf[NR], N1[NR], F2[NR];
                // KF = column slot of f (compile-time in each branch); the mask word of r0 is handled
                // by data: clr[w] is bit r0 in its own word and 0 in the other
                u64 clr[NR];
#pragma unroll
                for (int w = 0; w < NR; ++w) clr[w] = (r0 >> 6) == w ? bit0 : 0ull;
                auto level1 = [&](auto KFc) {
                    constexpr int KF = decltype(KFc)::value;
#pragma unroll
                    for (int w = 0; w < NR; ++w) {
                        cmf[w] = rdl64(cm[KF][w], f & 63) & ~clr[w];
                        wrlane64(cm[KF][w], cmf[w], f & 63);
                    }
#pragma unroll
                    for (int k = 0; k < NR; ++k) {
                        u64 t = 0;
#pragma unroll
                        for (int w = 0; w < NR; ++w) t |= cm[k][w] & clr[w];
                        N1[k] = ballot(t != 0);
                    }
                };
                if constexpr (NR == 2) {
                    if ((f >> 6) == 0) level1(std::integral_constant<int, 0>{});
                    else level1(std::integral_constant<int, 1>{});
                } else {
                    level1(std::integral_constant<int, 0>{});
                }
                // every row is matched here (r0 nominally), so no "unmatched" test is needed
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    const int m = mr[k];
                    u64 t;
                    if constexpr (NR == 2) t = (m & 64) ? (N1[1] >> (m & 63)) : (N1[0] >> (m & 63));
                    else t = N1[0] >> (m & 63);
                    F2[k] = ballot((t & 1) != 0);
                }
                u64 c2[NR];
#pragma unroll
                for (int w = 0; w < NR; ++w) c2[w] = cmf[w] & F2[w];
                if (__builtin_expect(any(c2), 1)) {
                    const int a1 = lowest(c2);
                    const int d1 = mr_of(a1);
                    set_mr(a1, f);
                    set_mr(r0, d1);
                } else {
                    bool done = false;
                    if (any(N1)) {
                        set_mr(r0, -1);
                        u64 N2[NR], F3[NR], c3[NR];
                        expand(F2, N2);
#pragma unroll
                        for (int w = 0; w < NR; ++w) N2[w] &= ~N1[w];
                        rows_matched_into(N2, F3);
#pragma unroll
                        for (int w = 0; w < NR; ++w) c3[w] = cmf[w] & F3[w];
                        if (any(c3)) {
                            const int a2 = lowest(c3);
                            const int d2 = mr_of(a2);
                            u64 cd[NR];
                            col_mask(d2, cd);
#pragma unroll
                            for (int w = 0; w < NR; ++w) cd[w] &= F2[w];
                            const int a1 = lowest(cd);
                            const int d1 = mr_of(a1);
                            set_mr(a2, f);
                            set_mr(a1, d2);
                            set_mr(r0, d1);
                            done = true;
                        }
                    }
                    if (!done) {
                        // deeper than three levels: let the general search redo it
                        set_mr(r0, -1);
#pragma unroll
                        for (int w = 0; w < NR; ++w)
                            if ((f >> 6) == w) FREEC[w] |= 1ull << (f & 63);
                        if (!augment(r0)) status = -3;     // leaves the loop before the sync
                    }
                }
            } else {
                // ---- general path: unmatch every exhausted cell first, then re-augment in order
                u64 z[NR];
#pragma unroll
                for (int w = 0; w < NR; ++w) z[w] = Z[w];
                while (any(z)) {
                    const int a = lowest(z);
                    const int d = mr_of(a);
                    const u64 bit = 1ull << (a & 63);
                    const bool here = lane == (d & 63);
#pragma unroll
                    for (int k = 0; k < NR; ++k) {
                        if ((d >> 6) == k) {
#pragma unroll
                            for (int w = 0; w < NR; ++w)
                                if ((a >> 6) == w) cm[k][w] = here ? cm[k][w] & ~bit : cm[k][w];
                            FREEC[k] |= 1ull << (d & 63);
                        }
                    }
#pragma unroll
                    for (int w = 0; w < NR; ++w)
                        if ((a >> 6) == w) z[w] &= ~bit;
                }
#pragma unroll
                for (int k = 0; k < NR; ++k) mr[k] = zero[k] ? -1 : mr[k];
                bool ok = true;
#pragma unroll
                for (int w = 0; w < NR; ++w)
                    for (u64 zz = Z[w]; zz && ok; zz &= zz - 1) ok = augment(64 * w + __builtin_ctzll(zz));
                if (!ok) status = -3;
            }
            if (__builtin_expect(status < 0, 0)) break;     // a row is unmatched: nothing to sync
            sync_matched(std::false_type{});
        }
        if (lane == 0) out_num[b] = status < 0 ? status : s;
    };
    if (narrow) run((u32)0);
    else run((u64)0);
}

// One wavefront per matrix: matrix blockIdx.x.  COST: the same wavefront goes on to evaluate the
// completion-time model of its matrix (kernel 3's body: a few reductions over what this kernel
// and kernel 1 left in memory), which saves a launch where launches are what a call costs;
// not available when that model needs the stage weights sorted.  A compile-time switch, so that
// the large-cluster instantiations are exactly the stage loop and nothing else.
template <int NR, bool FULL, bool COST>
__global__ void __launch_bounds__(K2_THREADS)
k2_birkhoff(const i64* __restrict__ wsQ, const i64* __restrict__ wsPart,
            int32_t* __restrict__ out_stages, i64* __restrict__ out_bytes,
            int32_t* __restrict__ out_num, i64* __restrict__ wsC, int S, int max_stages,
            const i64* __restrict__ wsT, double* __restrict__ out_time, int G, double bw_up,
            double bw_out, double delay) {
    extern __shared__ __align__(16) unsigned char k2_smem[];
    k2_matrix<NR, FULL>(wsQ, wsPart, out_stages, out_bytes, out_num, wsC, S, max_stages,
                        (int)blockIdx.x, (int)threadIdx.x, k2_smem);
    if constexpr (COST) {
        wave_sync();        // the stage count and the stage weights were stored by this wavefront
        k3_matrix<K2_THREADS>(wsT, wsPart, wsC, out_num, out_time, S, G, max_stages, bw_up, bw_out,
                              delay, 0, (int)blockIdx.x, (int)threadIdx.x, nullptr);
    }
}

}  // namespace fastk
