// Kernel 2: embedding and Birkhoff decomposition of the server-level matrix.
//
// One wavefront (64 lanes) per traffic matrix.  The stage loop of Birkhoff's
// decomposition (paper Section 4.4 "Birkhoff's decomposition: overview") is a
// chain of dependent steps - find a perfect matching, take the smallest matched
// entry as the stage weight, subtract, repair the matching - and a generic
// matrix needs about (S-1)^2 stages, so the design goal is the fewest
// instructions per stage, not memory throughput: a lone wavefront issues one
// instruction every four cycles at best, whatever its kind, and waits out every
// dependency on top of that.
//   * a single wavefront owns the matrix, so no step needs a workgroup barrier;
//     lane l owns rows l, l+64 and columns l, l+64 (S <= 128);
//   * the residual matrix R = Q + A lives in LDS (8-byte cells, odd row stride so
//     that a column - one cell per lane - spreads over the banks).  The residual of
//     each row's matched cell is also held in a register; after every subtraction
//     the register is written back, so LDS is current for every cell;
//   * almost every stage exhausts exactly one cell (r0, f).  The canonical search
//     then looks, on its second level, for the lowest row a1 that has a positive
//     cell in the unmatched column f and whose own column d1 has a positive cell
//     in row r0.  Both conditions are reads of R: every lane reads R[its row][f]
//     and R[r0][its column], a ballot of "both positive" gives the candidate rows,
//     and the two cells read by a1's lane are exactly the cells that get matched
//     next (a1 takes (a1, f), r0 takes (r0, d1)), so the repair and the reload of
//     the two re-matched rows cost one LDS round trip and no bit-mask work;
//   * the support of R as one S-bit row mask per column is what the deeper
//     repairs and the general search work on.  It is kept in LDS, where the stage
//     loop clears one bit per exhausted cell with an LDS atomic that nothing
//     waits for, and loaded into registers only by the repairs that search:
//     frontiers, visited sets and the set of unmatched columns are wave-uniform
//     bit masks, one breadth-first level is a few AND/compare operations per lane
//     plus ballots, parents are recomputed while the augmenting path is flipped;
//   * the stages that end in such a two-level repair run in an inner loop of
//     their own; everything else (several cells exhausted at once, a repair of
//     three levels or more, the end) leaves it with a reason.  Keeping the common
//     case a loop with a single back edge is what keeps the compiler from
//     shuffling the loop-carried registers at every merge;
//   * the virtual matrix A of the embedding (Section 4.4 "Adapting an arbitrary
//     matrix to a valid form") is never stored: pouring row deficits into column
//     deficits in ascending order makes A[a][d] the overlap of two prefix-sum
//     intervals (plus the diagonal term);
//   * no residual exceeds L, the largest row/column sum.  When L < 2^31 - directly, or
//     after a power of two common to all entries has been divided out - a cell of R
//     is two 32-bit halves, the residual and the real bytes left in it; the
//     write-back stores both (one 64-bit store), the reads of the repair return both,
//     and the stage loop runs on 32-bit registers with nothing to recompute when a
//     cell that holds virtual bytes gets matched (on skewed traffic, where most of L
//     is virtual, that is every third stage).  Otherwise a cell is one 64-bit word
//     with the top bit set where it holds virtual bytes, and the overlap is
//     recomputed when such a cell gets matched; the real bytes left in a cell never
//     exceed the largest entry of Q, so they are counted in 32 bits whenever that
//     fits;
//   * when S fills the lane slots exactly (64 or 128) the stage loop carries no
//     bounds predicates.  Predicated LDS writes and mid-loop exits cost a lone
//     wavefront far more than their instruction count suggests, so the stage avoids
//     them: unconditional write-back, the stage weight stored by every lane;
//   * LDS instructions complete in order and the compiler's wait for the reads of
//     the repair also waits for whatever was issued after them, so the atomic that
//     clears the support bit is issued once the reads have been consumed, and only
//     one lane sends it to the mask word (the other lanes to a word of their own): 64
//     lanes on one word are 64 serial passes that the next stage's LDS traffic would
//     queue behind.  That lane is the one holding the exhausted row: word and bit
//     follow from constants of its own and its column;
//   * every instruction of the stage costs the lone wavefront three to six clocks
//     wherever it sits, so nothing is spent on waiting by s_nop: the two instructions
//     the hardware wants between dependent DPP steps of the minimum are the part of
//     the previous stage's repair that the minimum does not need (new columns and
//     real-byte counts of the two re-matched rows; only their residuals are merged
//     first) and the advance of the store offsets.
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

// LDS: R[S][row stride], column deficit intervals PC[S], EC[S], frontier history [(S+2)][2].
// Row stride of R in words: odd, so that a column of the matrix (one cell per lane, read when
// a row looks for its cell in the unmatched column) falls into different LDS banks.
__host__ __device__ inline int k2_row_stride(int S) { return S | 1; }
__host__ __device__ inline size_t k2_lds_data_bytes(int S) {
    return (size_t)S * k2_row_stride(S) * 8 + (size_t)2 * S * 8 + (size_t)(S + 2) * 16;
}

// ... plus a spare region that the lane slots without a row (S below 64 * NR) read and write
// instead of a row of R, so that the stage loop needs no bounds predicate, plus the support
// masks: one 128-bit row mask per column, plus one word per lane for the lanes that take no
// part in a mask update
__host__ __device__ inline size_t k2_lds_spare_bytes(int S) { return (size_t)(S + 2) * 8; }
inline size_t k2_lds_bytes(int S) {
    return k2_lds_data_bytes(S) + k2_lds_spare_bytes(S) + (size_t)128 * 16 + 256;
}

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
    const int RS = k2_row_stride(S);
    i64* PC = reinterpret_cast<i64*>(R + (size_t)S * RS);
    i64* EC = PC + S;
    u64* Fh = reinterpret_cast<u64*>(EC + S);       // [level][2]

    i64 diag[NR], PR[NR], ER[NR];
    i64 qmax = 0;
    int sh = 0;         // every byte count below is in units of 2^sh bytes (0 unless that makes L fit 31 bits)
    const i64 L = embed_into_lds<NR, true>(wsQ, wsPart, b, S, RS, lane, R, PC, EC, diag, PR, ER, qmax, sh);
    if (L <= 0) {
        if (lane == 0) out_num[b] = (int32_t)L;     // -1: invalid input, 0: nothing to send
        return;
    }

    // Residuals never exceed L: when L < 2^31 the embedding has left cells of two 32-bit halves
    // (residual, real bytes left) and the stage loop runs on 32-bit registers.
    const bool narrow = L < ((i64)1 << 31);
    // support masks: bit a of cm[k][a/64] set while R[a][column lane+64k] > 0
    u64 cm[NR][NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int x = lane + 64 * k;
#pragma unroll
        for (int w = 0; w < NR; ++w) cm[k][w] = 0;
        if (x < S) {
            for (int a = 0; a < S; ++a) {
                const u64 w0 = R[a * RS + x];
                const u64 pos = narrow ? (u32)w0 != 0 : (w0 & ~VFLAG) != 0;
#pragma unroll
                for (int w = 0; w < NR; ++w)
                    if ((a >> 6) == w) cm[k][w] |= pos << (a & 63);
            }
        }
    }

    // Residuals never exceed L, so when L < 2^31 the whole stage loop runs on 32-bit words: the
    // residual matrix is repacked in place (flag in bit 31) and every per-stage subtraction,
    // comparison and select is one instruction instead of two.
    auto run = [&](auto tag, auto rltag, auto pairtag) {
        typedef decltype(tag) V;                // word type of the residuals
        typedef std::make_signed_t<V> SV;
        typedef decltype(rltag) RL;             // signed type of the real bytes left in a cell
        constexpr i64 RL_MAX = (i64)std::numeric_limits<RL>::max();
        constexpr V VF = (V)((V)1 << (sizeof(V) * 8 - 1));   // the cell holds virtual bytes
        // PAIRS: a cell of R is {low: residual, high: real bytes left}, kept current by the
        // write-back; otherwise one word, top bit set where the cell holds virtual bytes
        constexpr bool PAIRS = decltype(pairtag)::value;
        typedef std::conditional_t<PAIRS, u64, V> CELL;
        CELL* Rv = reinterpret_cast<CELL*>(k2_smem);
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
            const u32 spare = (u32)(k2_lds_data_bytes(S) / sizeof(CELL)) + 1u;
            rowbase[k] = lane + 64 * k < S ? (u32)(lane + 64 * k) * (u32)RS : spare;
        }
        int mr[NR], loaded[NR];
        SV rv[NR];
        RL rl[NR];
        u32 vfl[NR];       // bit 31: the matched cell holds virtual bytes (the flag of its LDS word)
        auto val_of = [&](CELL x) -> V {
            if constexpr (PAIRS) return (V)(u32)x;
            else return x & (V)~VF;
        };
        auto real_of = [&](CELL x) -> RL {      // where the cell holds no virtual bytes
            if constexpr (PAIRS) return (RL)(u32)(x >> 32);
            else return (RL)(x & (V)~VF);
        };
        auto with_flag = [&](SV v, u32 fl) -> V {
            if constexpr (sizeof(V) == 8) return (V)v | ((V)fl << 32);
            else return (V)v | fl;
        };
        auto cell_of = [&](SV v, RL real, u32 fl) -> CELL {
            if constexpr (PAIRS) return (u64)(u32)v | ((u64)(u32)real << 32);
            else return with_flag(v, fl);
        };
        auto flag_of = [&](CELL x) -> u32 {
            if constexpr (PAIRS) return 0u;
            else if constexpr (sizeof(V) == 8) return (u32)(x >> 32) & 0x80000000u;
            else return (u32)x & 0x80000000u;
        };
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
            CELL x[NR];
            bool ch[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                ch[k] = mr[k] != loaded[k];
                if constexpr (PLAIN) {
                    Rv[rowbase[k] + (u32)loaded[k]] = cell_of(rv[k], rl[k], vfl[k]);
                    x[k] = Rv[rowbase[k] + (u32)mr[k]];
                } else {
                    if (ch[k] && rv[k] > 0) Rv[rowbase[k] + (u32)loaded[k]] = cell_of(rv[k], rl[k], vfl[k]);
                    x[k] = Rv[rowbase[k] + (u32)max(mr[k], 0)];
                }
            }
            u64 anyv = 0;
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const V val = val_of(x[k]);
                const u32 fl = flag_of(x[k]);
                rv[k] = ch[k] ? (SV)val : rv[k];
                rl[k] = ch[k] ? real_of(x[k]) : rl[k];
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
                        rl[k] = (i64)rv[k] > av ? (RL)((i64)rv[k] - av) : (RL)0;
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

        // The support masks also live in LDS, one 128-bit row mask per column: the stage loop
        // clears bits there (one LDS atomic, nothing waits for it) and only the repairs that
        // need a search load them back into registers.
        u64* cmL = reinterpret_cast<u64*>(k2_smem + k2_lds_data_bytes(S) + k2_lds_spare_bytes(S));
        auto masks_to_lds = [&]() {
#pragma unroll
            for (int k = 0; k < NR; ++k)
#pragma unroll
                for (int w = 0; w < 2; ++w) cmL[(lane + 64 * k) * 2 + w] = w < NR ? cm[k][w < NR ? w : 0] : 0ull;
        };
        auto masks_from_lds = [&]() {
#pragma unroll
            for (int k = 0; k < NR; ++k)
#pragma unroll
                for (int w = 0; w < NR; ++w) cm[k][w] = cmL[(lane + 64 * k) * 2 + w];
        };
        masks_to_lds();
        u64 LIVE[NR];      // lane slots that hold a row
#pragma unroll
        for (int k = 0; k < NR; ++k) LIVE[k] = ballot(lane + 64 * k < S);

        int32_t* stg = out_stages + (size_t)b * max_stages * S;
        i64* byt = out_bytes + (size_t)b * max_stages * S;
        i64* cw = wsC + (size_t)b * max_stages;
        std::conditional_t<PAIRS, u32, i64> Lrem = (std::conditional_t<PAIRS, u32, i64>)L;
        int s = 0;
        // byte offsets of the lane's first slot in the stage row being written
        u32 soff = (u32)lane * 4u, boff = (u32)lane * 8u, coff = 0;
        asm volatile("" : "+v"(coff));     // a vector register of its own: the store needs one anyway
        // DEFER (two-half cells): the DPP steps of the stage-weight minimum
        // need two instructions between them; instead of s_nop those are the part of the previous
        // stage's repair that the minimum does not depend on - the new columns and the new
        // real-byte counts of the two re-matched rows - and the advance of the three store
        // offsets, which therefore name the stage before the one being emitted until then.
        constexpr bool DEFER = PAIRS;
        const u32 stride_s = 4u * (u32)S, stride_b = 8u * (u32)S;
        if constexpr (DEFER) { soff -= stride_s; boff -= stride_b; coff -= 8u; }
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

        // cell (a, d) has left the support (a, d wave-uniform): one LDS atomic that nothing waits
        // for; every lane sends the same AND to the same word (written as an instruction of its
        // own: the compiler would wrap an atomicAnd into a dozen instructions that pick one lane)
        const u32 dummy_addr = (u32)(k2_lds_data_bytes(S) + k2_lds_spare_bytes(S)) + 128u * 16u + (u32)lane * 4u;
        u32 mbase[NR], mkeep[NR];      // word (for column 0) and bit of the lane's rows in the masks
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            mbase[k] = (u32)(k2_lds_data_bytes(S) + k2_lds_spare_bytes(S)) + (u32)(lid[k] >> 5) * 4u;
            mkeep[k] = ~(1u << (lid[k] & 31));
        }
        auto clear_edge = [&](int a, int d) {
            // lane 0 clears the bit; the other lanes send theirs to a word of their own behind the
            // masks (64 lanes on one word would be 64 serial passes through the LDS pipeline)
            const u32 real = (u32)(k2_lds_data_bytes(S) + k2_lds_spare_bytes(S)) +
                             (u32)d * 16u + (u32)(a >> 5) * 4u;
            const u32 addr = lane == 0 ? real : dummy_addr;
            const u32 keep = ~(1u << (a & 31));
            asm volatile("ds_and_b32 %0, %1" : : "v"(addr), "v"(keep) : "memory");
        };
        // LDS follows every subtraction: each row's matched cell gets its new residual (the
        // exhausted one its zero), so that R in LDS is current for every cell.  Where it sits in
        // the stage is a matter of measurement: before the reads of the repair when a lane holds
        // two rows, after them (with the one stale cell masked out) when it holds one.
        constexpr bool LATE_WRITE_BACK = NR == 1;
        auto write_back = [&]() {
#pragma unroll
            for (int k = 0; k < NR; ++k) Rv[rowbase[k] + (u32)mr[k]] = cell_of(rv[k], rl[k], vfl[k]);
        };
        // x of the lane slot that holds row a (a wave-uniform), as a wave-uniform value
        auto value_of_row = [&](const CELL (&x)[NR], int a) -> CELL {
            if constexpr (NR == 2) {
                if constexpr (sizeof(CELL) == 8) {
                    const u64 b0 = rdl64((u64)x[0], a & 63), b1 = rdl64((u64)x[1], a & 63);
                    return (CELL)((a & 64) ? b1 : b0);
                } else {
                    const u32 b0 = rdl((u32)x[0], a & 63), b1 = rdl((u32)x[1], a & 63);
                    return (CELL)((a & 64) ? b1 : b0);
                }
            } else {
                if constexpr (sizeof(CELL) == 8) return (CELL)rdl64((u64)x[0], a);
                else return (CELL)rdl((u32)x[0], a);
            }
        };
        // a cell's word without its flag bit, folded to 32 bits: non-zero while the cell is positive
        auto fold = [&](CELL x) -> u32 {
            if constexpr (PAIRS) return (u32)x;
            else if constexpr (sizeof(V) == 8) return ((u32)((u64)x >> 32) & 0x7FFFFFFFu) | (u32)x;
            else return (u32)x & 0x7FFFFFFFu;
        };
        // Whether a three-level repair is worked out from the reads of the stage plus one more
        // column read, or on the support masks alone: measured, the first wins when a lane holds
        // two rows and loses when it holds one.
        constexpr bool DEEP_FROM_READS = NR == 2;
        constexpr bool PAIR_FROM_READS = NR == 2;
        enum { GO_ON = 0, GENERAL, DEEP };
        for (;;) {
            // ---- the stages that end in a two-level repair run in this inner loop; anything
            // else leaves it with a reason and is handled below
            int why = GO_ON;
            u64 Z[NR];
            bool zero[NR];
            int r0 = 0, f = 0, nz = 0;
            CELL ea[NR], eb[NR];      // R[row][f] and R[r0][column of the row], read by the stage that left
#pragma unroll
            for (int k = 0; k < NR; ++k) ea[k] = eb[k] = 0;
            if (__builtin_expect(s >= max_stages, 0)) { status = -2; break; }
            // DEFER: what the previous stage of this run left to do (nothing at first)
            u64 pmA[NR], pmR[NR];
            int pf = 0, pd1 = 0;
            u32 pvh = 0;
#pragma unroll
            for (int k = 0; k < NR; ++k) pmA[k] = pmR[k] = 0;
            do {
                V mine = (V)rv[0];
                if constexpr (NR == 2) mine = (V)rv[1] < mine ? (V)rv[1] : mine;
                i64 c64;
                if constexpr (DEFER && NR == 1) {
                    // one row per lane: ten instructions for the seven gaps, s_nop for the rest
                    u32 v = (u32)mine, tf, td, th;
                    u32 m0 = (u32)mr[0], l0 = (u32)rl[0];
                    const u32 eh0 = (u32)((u64)ea[0] >> 32);
                    asm volatile(
                        "v_mov_b32 %[tf], %[pf]\n\t"
                        "v_mov_b32 %[td], %[pd1]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[m0], %[m0], %[td], %[mR0]\n\t"
                        "v_mov_b32 %[th], %[pvh]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[m0], %[m0], %[tf], %[mA0]\n\t"
                        "v_add_u32 %[soff], %[ds], %[soff]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[l0], %[l0], %[eh0], %[mA0]\n\t"
                        "v_add_u32 %[boff], %[db], %[boff]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] row_mirror row_mask:0xf bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[l0], %[l0], %[th], %[mR0]\n\t"
                        "v_add_u32 %[coff], 8, %[coff]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                        "s_nop 1\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                        "s_nop 1"
                        : [v] "+v"(v), [tf] "=&v"(tf), [td] "=&v"(td), [th] "=&v"(th), [m0] "+v"(m0),
                          [l0] "+v"(l0), [soff] "+v"(soff), [boff] "+v"(boff), [coff] "+v"(coff)
                        : [pf] "s"(pf), [pd1] "s"(pd1), [pvh] "s"(pvh), [mR0] "s"(pmR[0]),
                          [mA0] "s"(pmA[0]), [eh0] "v"(eh0), [ds] "s"(stride_s), [db] "s"(stride_b));
                    mr[0] = (int)m0;
                    rl[0] = (RL)l0;
                    c64 = (i64)rdl(v, 63);
                } else if constexpr (DEFER) {
                    u32 v = (u32)mine, tf, td;
                    u32 m0 = (u32)mr[0], m1 = (u32)mr[NR - 1], l0 = (u32)rl[0], l1 = (u32)rl[NR - 1];
                    const u32 eh0 = (u32)((u64)ea[0] >> 32), eh1 = (u32)((u64)ea[NR - 1] >> 32);
                    asm volatile(
                        "v_mov_b32 %[tf], %[pf]\n\t"
                        "v_mov_b32 %[td], %[pd1]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[m0], %[m0], %[td], %[mR0]\n\t"
                        "v_cndmask_b32_e64 %[m1], %[m1], %[td], %[mR1]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[m0], %[m0], %[tf], %[mA0]\n\t"
                        "v_cndmask_b32_e64 %[m1], %[m1], %[tf], %[mA1]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                        "v_mov_b32 %[tf], %[pvh]\n\t"
                        "v_add_u32 %[soff], %[ds], %[soff]"
                        : [v] "+v"(v), [tf] "=&v"(tf), [td] "=&v"(td), [m0] "+v"(m0), [m1] "+v"(m1),
                          [soff] "+v"(soff)
                        : [pf] "s"(pf), [pd1] "s"(pd1), [pvh] "s"(pvh), [mR0] "s"(pmR[0]),
                          [mR1] "s"(pmR[NR - 1]), [mA0] "s"(pmA[0]), [mA1] "s"(pmA[NR - 1]),
                          [ds] "s"(stride_s));
                    asm volatile(
                        "v_min_u32_dpp %[v], %[v], %[v] row_mirror row_mask:0xf bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[l0], %[l0], %[eh0], %[mA0]\n\t"
                        "v_cndmask_b32_e64 %[l1], %[l1], %[eh1], %[mA1]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                        "v_cndmask_b32_e64 %[l0], %[l0], %[th], %[mR0]\n\t"
                        "v_cndmask_b32_e64 %[l1], %[l1], %[th], %[mR1]\n\t"
                        "v_min_u32_dpp %[v], %[v], %[v] row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
                        "v_add_u32 %[boff], %[db], %[boff]\n\t"
                        "v_add_u32 %[coff], 8, %[coff]"
                        : [v] "+v"(v), [l0] "+v"(l0), [l1] "+v"(l1), [boff] "+v"(boff), [coff] "+v"(coff)
                        : [th] "v"(tf), [eh0] "v"(eh0), [eh1] "v"(eh1), [mA0] "s"(pmA[0]),
                          [mA1] "s"(pmA[NR - 1]), [mR0] "s"(pmR[0]), [mR1] "s"(pmR[NR - 1]),
                          [db] "s"(stride_b));
                    mr[0] = (int)m0;
                    mr[NR - 1] = (int)m1;
                    rl[0] = (RL)l0;
                    rl[NR - 1] = (RL)l1;
                    c64 = (i64)rdl(v, 63);
                } else {
                    c64 = (i64)wave_min(mine);      // stage weight: wave-uniform, fits SV
                }
                // one copy of the weight in vector registers for all the per-lane arithmetic
                SV c;
                if constexpr (sizeof(V) == 8) {
                    u32 clo, chi;
                    asm volatile("v_mov_b32 %0, %2\n\tv_mov_b32 %1, %3"
                                 : "=v"(clo), "=v"(chi) : "s"((u32)c64), "s"((u32)((u64)c64 >> 32)));
                    c = (SV)(((u64)chi << 32) | clo);
                } else {
                    u32 clo;
                    asm volatile("v_mov_b32 %0, %1" : "=v"(clo) : "s"((u32)c64));
                    c = (SV)clo;
                }
                RL cr;
                if constexpr (sizeof(RL) == sizeof(SV)) cr = (RL)c;
                else cr = (RL)(c64 < RL_MAX ? c64 : RL_MAX);
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    const RL real = cr < rl[k] ? cr : rl[k];
                    rl[k] -= real;
                    rv[k] -= c;
                    if (FULL || lid[k] < S) {
                        *reinterpret_cast<int32_t*>(reinterpret_cast<char*>(stg) + soff + 256u * k) =
                            real > 0 ? mr[k] : -1;
                        *reinterpret_cast<i64*>(reinterpret_cast<char*>(byt) + boff + 512u * k) =
                            (i64)(std::make_unsigned_t<RL>)real << sh;
                    }
                    zero[k] = rv[k] == 0;
                    Z[k] = ballot(zero[k]);
                }
                // every lane stores the same word: no divergent branch on the path
                *reinterpret_cast<i64*>(reinterpret_cast<char*>(cw) + coff) = (i64)(std::make_unsigned_t<SV>)c << sh;
                ++s;
                if constexpr (!DEFER) {
                    soff += stride_s;
                    boff += stride_b;
                    coff += 8u;
                }
                Lrem -= (std::conditional_t<PAIRS, u32, i64>)c64;
                // (the stage that ends the decomposition leaves every row at zero: it takes the
                // exit for several exhausted cells below and is told apart after the loop)
                if constexpr (!LATE_WRITE_BACK) write_back();
                nz = 0;
#pragma unroll
                for (int w = 0; w < NR; ++w) nz += __builtin_popcountll(Z[w]);
                if (__builtin_expect(nz != 1, 0)) { why = GENERAL; break; }
                // one exhausted cell (r0, f); f is the only unmatched column.  A two-level repair
                // takes the lowest row a1 that has a positive cell in column f and whose column
                // d1 has a positive cell in row r0: both tests are reads of R, and the two cells
                // read by a1's lane are the ones that get matched.
                if constexpr (NR == 2) {
                    const int ln = __builtin_ctzll(Z[0] | Z[1]);
                    r0 = ln | (Z[0] ? 0 : 64);
                    f = (int)rdl((u32)(zero[0] ? mr[0] : mr[1]), ln);
                } else {
                    r0 = lowest(Z);
                    f = mr_of(r0);
                }
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    ea[k] = Rv[rowbase[k] + (u32)f];
                    eb[k] = Rv[(u32)r0 * (u32)RS + (u32)(FULL ? mr[k] : max(mr[k], 0))];
                }
                if constexpr (LATE_WRITE_BACK) write_back();
                u64 c2[NR];
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    // both cells positive: fold each to 32 bits, take the smaller
                    c2[k] = ballot(min(fold(ea[k]), fold(eb[k])) != 0);
                    if constexpr (LATE_WRITE_BACK)
                        if ((r0 >> 6) == k) c2[k] &= ~(1ull << (r0 & 63));     // its cell (r0, f) was read stale
                    if constexpr (!FULL) c2[k] &= LIVE[k];
                }
                {   // issued once the reads have been consumed (the unused operand pins it behind
                    // the candidate masks): nothing waits for it
                    u32 addr, keep;
                    if constexpr (NR == 2) {
                        // the lane that holds the exhausted row knows the word and the bit from
                        // constants of its own and its column; the other lanes go to their dummies
                        addr = zero[1] ? ((u32)mr[1] << 4) + mbase[1] : dummy_addr;
                        addr = zero[0] ? ((u32)mr[0] << 4) + mbase[0] : addr;
                        keep = zero[0] ? mkeep[0] : mkeep[1];
                    } else {
                        addr = zero[0] ? ((u32)mr[0] << 4) + mbase[0] : dummy_addr;
                        keep = mkeep[0];
                    }
                    u64 dep = c2[0];
                    if constexpr (NR == 2) dep |= c2[1];
                    asm volatile("ds_and_b32 %0, %1" : : "v"(addr), "v"(keep), "s"(dep) : "memory");
                }
                if (__builtin_expect(!any(c2), 0)) { why = DEEP; break; }
                const int a1 = lowest(c2);
                int d1;
                CELL vb;
                if constexpr (NR == 2) {
                    // pick the slot first, then one readlane per word
                    const bool up = c2[0] == 0;
                    d1 = (int)rdl((u32)(up ? mr[1] : mr[0]), a1 & 63);
                    vb = (CELL)rdl64((u64)(up ? eb[1] : eb[0]), a1 & 63);
                } else {
                    d1 = mr_of(a1);
                    vb = value_of_row(eb, a1);
                }
                u64 anyv = 0;
                if constexpr (DEFER) {
                    // the residuals now (the next minimum needs them), the rest during that minimum
#pragma unroll
                    for (int k = 0; k < NR; ++k) {
                        // (row r0 is the one row at zero: its mask is at hand)
                        const bool isA = lid[k] == a1;
                        const u32 xa = isA ? (u32)(u64)ea[k] : (u32)rv[k];
                        rv[k] = zero[k] ? (SV)(u32)(u64)vb : (SV)xa;
                        pmA[k] = ballot(isA);
                        pmR[k] = Z[k];
                    }
                    pf = f;
                    pd1 = d1;
                    pvh = (u32)((u64)vb >> 32);
                } else {
#pragma unroll
                for (int k = 0; k < NR; ++k) {
                    const bool isA = lid[k] == a1, isR = lid[k] == r0;
                    const CELL x = isA ? ea[k] : vb;
                    const bool ch = isA || isR;
                    const V val = val_of(x);
                    const u32 fl = flag_of(x);
                    rv[k] = ch ? (SV)val : rv[k];
                    rl[k] = ch ? real_of(x) : rl[k];
                    vfl[k] = ch ? fl : vfl[k];
                    anyv |= (ballot(isA) | ballot(isR)) & ballot(flag_of(x) != 0);
                    mr[k] = isA ? f : (isR ? d1 : mr[k]);
                }
                }
                if (__builtin_expect(anyv != 0, 0)) {
#pragma unroll
                    for (int k = 0; k < NR; ++k) {
                        if ((lid[k] == a1 || lid[k] == r0) && vfl[k] != 0) {
                            const int d = mr[k];
                            const i64 l = max(PR[k], PC[d]);
                            const i64 h = min(ER[k], EC[d]);
                            const i64 av = (h > l ? h - l : 0) + (d == lid[k] ? diag[k] : 0);
                            rl[k] = (i64)rv[k] > av ? (RL)((i64)rv[k] - av) : (RL)0;
                        }
                    }
                }
            } while (__builtin_expect(s < max_stages, 1));
            if (Lrem == 0) break;                           // done
            if (why == GO_ON) { status = -2; break; }       // out of stage rows
#pragma unroll
            for (int k = 0; k < NR; ++k) loaded[k] = mr[k];     // what LDS and the registers describe
            if (why == DEEP) {
                if constexpr (DEEP_FROM_READS) {
                    // Not a two-level repair.  Level three, still in straight-line code: the reads of
                    // the stage say which rows have a cell in column f (cmf) and which are matched
                    // into a column that row r0 reaches (F2, the second frontier); the support masks
                    // give the columns that F2 reaches (N2) and with them the third frontier; the
                    // lowest of its rows with a cell in column f is a2, and one more column read
                    // finds a2's parent a1 in F2 - and is the cell a1 gets matched to.
                    u64 cmf[NR], F2[NR];
#pragma unroll
                    for (int k = 0; k < NR; ++k) {
                        const u64 notr0 = (r0 >> 6) == k ? ~(1ull << (r0 & 63)) : ~0ull;
                        cmf[k] = ballot(fold(ea[k]) != 0) & notr0;
                        F2[k] = ballot(fold(eb[k]) != 0) & notr0;
                        if constexpr (!FULL) { cmf[k] &= LIVE[k]; F2[k] &= LIVE[k]; }
                    }
                    masks_from_lds();
                    bool done = false;
                    if (any(F2)) {
                        u64 N2[NR], F3[NR], c3[NR];
                        expand(F2, N2);
                        rows_matched_into(N2, F3);
                        // rows matched into a column that r0 reaches itself are on level two already
#pragma unroll
                        for (int w = 0; w < NR; ++w) c3[w] = cmf[w] & F3[w] & ~F2[w];
                        if (any(c3)) {
                            const int a2 = lowest(c3);
                            const int d2 = mr_of(a2);
                            CELL ec[NR];
                            u64 c1[NR];
#pragma unroll
                            for (int k = 0; k < NR; ++k) {
                                ec[k] = Rv[rowbase[k] + (u32)d2];
                                c1[k] = F2[k] & ballot(fold(ec[k]) != 0);
                            }
                            if (any(c1)) {
                                const int a1 = lowest(c1);
                                const int d1 = mr_of(a1);
                                const CELL vb = value_of_row(eb, a1);
                                u64 anyv = 0;
#pragma unroll
                                for (int k = 0; k < NR; ++k) {
                                    const bool isA2 = lid[k] == a2, isA1 = lid[k] == a1, isR = lid[k] == r0;
                                    const CELL x = isA2 ? ea[k] : (isA1 ? ec[k] : vb);
                                    const bool ch = isA2 || isA1 || isR;
                                    const V val = val_of(x);
                                    const u32 fl = flag_of(x);
                                    rv[k] = ch ? (SV)val : rv[k];
                                    rl[k] = ch ? real_of(x) : rl[k];
                                    vfl[k] = ch ? fl : vfl[k];
                                    anyv |= ballot(ch && fl != 0);
                                    mr[k] = isA2 ? f : (isA1 ? d2 : (isR ? d1 : mr[k]));
                                }
                                if (anyv != 0) {
#pragma unroll
                                    for (int k = 0; k < NR; ++k) {
                                        if ((lid[k] == a2 || lid[k] == a1 || lid[k] == r0) && vfl[k] != 0) {
                                            const int d = mr[k];
                                            const i64 l = max(PR[k], PC[d]);
                                            const i64 h = min(ER[k], EC[d]);
                                            const i64 av = (h > l ? h - l : 0) + (d == lid[k] ? diag[k] : 0);
                                            rl[k] = (i64)rv[k] > av ? (RL)((i64)rv[k] - av) : (RL)0;
                                        }
                                    }
                                }
                                done = true;
                            }
                        }
                    }
                    if (done) continue;     // LDS and the registers agree: on to the next stage
                    // deeper than three levels: let the general search redo it
                    set_mr(r0, -1);
#pragma unroll
                    for (int w = 0; w < NR; ++w)
                        if ((f >> 6) == w) FREEC[w] |= 1ull << (f & 63);
                    if (!augment(r0)) status = -3;
                } else {
                    // not a two-level repair: level three in straight-line code on the masks,
                    // anything deeper through the general search
                    masks_from_lds();
                    const u64 bit0 = 1ull << (r0 & 63);
                    u64 cmf[NR], N1[NR], F2[NR];
                    col_mask(f, cmf);
                    {
                        u64 F1[NR];
#pragma unroll
                        for (int w = 0; w < NR; ++w) F1[w] = (r0 >> 6) == w ? bit0 : 0ull;
                        expand(F1, N1);
                        rows_matched_into(N1, F2);
                    }
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
                        if (!augment(r0)) status = -3;
                    }
                }
            } else {
                // ---- several exhausted cells: all of them are unmatched first, then the rows are
                // re-augmented in ascending order.  Two cells (rA, fA), (rB, fB) with rA < rB - by far
                // the most frequent case - are repaired like the single cell, on reads of R, as long
                // as each row's augmenting path has one or two levels: rA takes fB if it has a cell
                // there, otherwise the lowest free column that its second frontier reaches; rB then
                // takes the column left over, directly or through the second frontier under the
                // matching as it stands by then.  Whatever that does not settle goes to the search.
                int pending = (PAIR_FROM_READS && nz == 2) ? 2 : 3;     // 0: repaired, 1: second row left to the search, 3: everything
                if (PAIR_FROM_READS && nz == 2) {
                    u64 zz[NR];
#pragma unroll
                    for (int w = 0; w < NR; ++w) zz[w] = Z[w];
                    const int rA = lowest(zz);
#pragma unroll
                    for (int w = 0; w < NR; ++w)
                        if ((rA >> 6) == w) zz[w] &= ~(1ull << (rA & 63));
                    const int rB = lowest(zz);
                    const int fA = mr_of(rA), fB = mr_of(rB);
                    if constexpr (LATE_WRITE_BACK) write_back();
                    clear_edge(rA, fA);
                    clear_edge(rB, fB);
                    CELL xa[NR], xb[NR], ya[NR];       // columns fA, fB; row rA along the matching
                    u64 others[NR];                 // rows that hold a matched cell
#pragma unroll
                    for (int k = 0; k < NR; ++k) {
                        xa[k] = Rv[rowbase[k] + (u32)fA];
                        xb[k] = Rv[rowbase[k] + (u32)fB];
                        ya[k] = Rv[(u32)rA * (u32)RS + (u32)(FULL ? mr[k] : max(mr[k], 0))];
                        others[k] = ~Z[k];
                        if constexpr (!FULL) others[k] &= LIVE[k];
                    }
                    bool chg[NR];
#pragma unroll
                    for (int k = 0; k < NR; ++k) chg[k] = false;
                    // row `row` (wave-uniform) is matched to column `col`, whose word in R is x
                    auto rematch = [&](int row, int col, CELL x) {
                        const V val = val_of(x);
                        const u32 fl = flag_of(x);
#pragma unroll
                        for (int k = 0; k < NR; ++k) {
                            const bool me = lid[k] == row;
                            rv[k] = me ? (SV)val : rv[k];
                            rl[k] = me ? real_of(x) : rl[k];
                            vfl[k] = me ? fl : vfl[k];
                            mr[k] = me ? col : mr[k];
                            chg[k] = chg[k] || me;
                        }
                    };
                    int fx = -1;                    // the column still free after the first row
                    const CELL yAB = value_of_row(ya, rB);     // R[rA][fB]: rB's register still names fB
                    if (fold(yAB) != 0) {
                        rematch(rA, fB, yAB);
                        fx = fA;
                    } else {
                        u64 ca[NR], cb[NR];         // second-frontier rows with a cell in fA / in fB
#pragma unroll
                        for (int k = 0; k < NR; ++k) {
                            const u64 F2 = ballot(fold(ya[k]) != 0) & others[k];
                            ca[k] = F2 & ballot(fold(xa[k]) != 0);
                            cb[k] = F2 & ballot(fold(xb[k]) != 0);
                        }
                        const bool ra = any(ca), rb = any(cb);
                        if (ra || rb) {
                            const bool takeA = ra && (!rb || fA < fB);      // the lower free column
                            int a1;
                            CELL va1;
                            if (takeA) { a1 = lowest(ca); va1 = value_of_row(xa, a1); }
                            else { a1 = lowest(cb); va1 = value_of_row(xb, a1); }
                            const int d1 = mr_of(a1);
                            const CELL vA = value_of_row(ya, a1);
                            rematch(a1, takeA ? fA : fB, va1);
                            rematch(rA, d1, vA);
                            fx = takeA ? fB : fA;
                        }
                    }
                    if (fx >= 0) {
                        pending = 1;
                        const bool isA = fx == fA;
                        const CELL xB = isA ? value_of_row(xa, rB) : value_of_row(xb, rB);     // R[rB][fx]
                        if (fold(xB) != 0) {
                            rematch(rB, fx, xB);
                            pending = 0;
                        } else {
                            CELL yb[NR];               // row rB along the matching as it is now
                            u64 c[NR];
#pragma unroll
                            for (int k = 0; k < NR; ++k) {
                                yb[k] = Rv[(u32)rB * (u32)RS + (u32)(FULL ? mr[k] : max(mr[k], 0))];
                                const CELL xk = isA ? xa[k] : xb[k];
                                u64 m = ballot(min(fold(yb[k]), fold(xk)) != 0);
                                if ((rB >> 6) == k) m &= ~(1ull << (rB & 63));
                                if constexpr (!FULL) m &= LIVE[k];
                                c[k] = m;
                            }
                            if (any(c)) {
                                const int a1 = lowest(c);
                                const int d1 = mr_of(a1);
                                const CELL va1 = isA ? value_of_row(xa, a1) : value_of_row(xb, a1);
                                const CELL vB = value_of_row(yb, a1);
                                rematch(a1, fx, va1);
                                rematch(rB, d1, vB);
                                pending = 0;
                            }
                        }
                        // re-matched cells that hold virtual bytes: what is left of their real bytes
#pragma unroll
                        for (int k = 0; k < NR; ++k) {
                            if (chg[k] && vfl[k] != 0 && mr[k] >= 0) {
                                const int d = mr[k];
                                const i64 l = max(PR[k], PC[d]);
                                const i64 h = min(ER[k], EC[d]);
                                const i64 av = (h > l ? h - l : 0) + (d == lid[k] ? diag[k] : 0);
                                rl[k] = (i64)rv[k] > av ? (RL)((i64)rv[k] - av) : (RL)0;
                            }
                        }
                        if (pending == 1) {
                            // the second row needs a longer path: the search takes it from here
#pragma unroll
                            for (int k = 0; k < NR; ++k) loaded[k] = mr[k];
                            set_mr(rB, -1);
#pragma unroll
                            for (int w = 0; w < NR; ++w)
                                if ((fx >> 6) == w) FREEC[w] |= 1ull << (fx & 63);
                            masks_from_lds();
                            if (!augment(rB)) status = -3;
                        }
                    }
                }
                if (pending == 0) continue;     // LDS and the registers agree: on to the next stage
                if (pending >= 2) {
                    u64 z[NR];
#pragma unroll
                    for (int w = 0; w < NR; ++w) z[w] = Z[w];
                    while (any(z)) {
                        const int a = lowest(z);
                        const int d = mr_of(a);
                        const u64 bit = 1ull << (a & 63);
                        clear_edge(a, d);
#pragma unroll
                        for (int k = 0; k < NR; ++k)
                            if ((d >> 6) == k) FREEC[k] |= 1ull << (d & 63);
#pragma unroll
                        for (int w = 0; w < NR; ++w)
                            if ((a >> 6) == w) z[w] &= ~bit;
                    }
                    masks_from_lds();
#pragma unroll
                    for (int k = 0; k < NR; ++k) mr[k] = zero[k] ? -1 : mr[k];
                    bool ok = true;
#pragma unroll
                    for (int w = 0; w < NR; ++w)
                        for (u64 zz = Z[w]; zz && ok; zz &= zz - 1) ok = augment(64 * w + __builtin_ctzll(zz));
                    if (!ok) status = -3;
                }
            }
            if (__builtin_expect(status < 0, 0)) break;     // a row is unmatched: nothing to sync
            sync_matched(std::false_type{});
        }
        if (lane == 0) out_num[b] = status < 0 ? status : s;
    };
    // the real bytes of a cell never exceed the largest entry of Q: 32-bit counters when that
    // fits, whatever the virtual bytes make of the residuals
    if (narrow) run((u32)0, (int32_t)0, std::true_type{});
    else if (qmax < ((i64)1 << 31)) run((u64)0, (int32_t)0, std::false_type{});
    else run((u64)0, (i64)0, std::false_type{});
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
