// Pieces shared by the two decomposition kernels (k2_birkhoff: the paper's rule, any perfect
// matching on the support; k9_bottleneck: a bottleneck assignment per stage): wavefront
// helpers, the embedding of the server-level matrix into LDS, and the canonical augmenting
// search on column masks.  One wavefront owns a matrix; lane l owns rows l, l+64 and columns
// l, l+64 (NR = 1 for S <= 64, 2 for S <= 128).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"

namespace fastk {

typedef unsigned int u32;

constexpr u64 VFLAG = 1ull << 63;      // LDS word flag: the cell holds virtual bytes

// Orders the LDS and global accesses of the one wavefront that owns a matrix (its lanes
// exchange data through memory).  Not a workgroup barrier: the decomposition code also runs as
// one wavefront of a larger workgroup, where the other wavefronts must not be waited for.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ u64 ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ u32 rdl(u32 v, int lane) { return (u32)__builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ u64 rdl64(u64 v, int lane) {
    return ((u64)rdl((u32)(v >> 32), lane) << 32) | rdl((u32)v, lane);
}

// tells the compiler that a value is the same in every lane
__device__ __forceinline__ u64 uniform64(u64 x) {
    return ((u64)(u32)__builtin_amdgcn_readfirstlane((u32)(x >> 32)) << 32) |
           (u64)(u32)__builtin_amdgcn_readfirstlane((u32)x);
}

// min over the 64 lanes (all lanes must be active), result wave-uniform
__device__ __forceinline__ u32 wave_min_u32(u32 v) {
    asm volatile(
        "s_nop 1\n\tv_min_u32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_min_u32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_min_u32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_min_u32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_min_u32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\tv_min_u32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(v));
    return rdl(v, 63);
}
__device__ __forceinline__ u64 wave_min_u64(u64 x) {
    const u32 hi = (u32)(x >> 32);
    // if some value fits 32 bits the minimum is among those: try that first, without a test
    // in front of the reduction (all-ones: none fits, or the minimum really is 2^32 - 1)
    const u32 first = wave_min_u32(hi == 0 ? (u32)x : 0xFFFFFFFFu);
    if (__builtin_expect(first != 0xFFFFFFFFu, 1)) return first;
    const u32 mhi = wave_min_u32(hi);
    const u32 lo = hi == mhi ? (u32)x : 0xFFFFFFFFu;
    const u32 mlo = wave_min_u32(lo);
    return ((u64)mhi << 32) | mlo;
}
// max over the 64 lanes (all lanes must be active), result wave-uniform
__device__ __forceinline__ u32 wave_max_u32(u32 v) {
    asm volatile(
        "s_nop 1\n\tv_max_u32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_max_u32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_max_u32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_max_u32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\tv_max_u32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\tv_max_u32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(v));
    return rdl(v, 63);
}
__device__ __forceinline__ u64 wave_max_u64(u64 x) {
    const u32 hi = (u32)(x >> 32);
    const u32 mhi = wave_max_u32(hi);
    const u32 lo = hi == mhi ? (u32)x : 0u;
    return ((u64)mhi << 32) | wave_max_u32(lo);
}
// v[lane] = val for one lane; val and lane are wave-uniform.  gfx950 lets v_writelane read one
// scalar register besides m0, so the lane index travels in m0; m0 is on the clobber list (the
// compiler reloads it before its own uses) and clang's warning that it is a reserved register,
// which it prints for any such clobber, is switched off for these two statements.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void wrlane(u32& v, u32 val, int lane) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tv_writelane_b32 %0, %1, m0"
                 : "+v"(v) : "s"(val), "s"(lane) : "m0");
}
__device__ __forceinline__ void wrlane64(u64& v, u64 val, int lane) {
    u32 lo = (u32)v, hi = (u32)(v >> 32);
    asm volatile("s_mov_b32 m0, %4\n\ts_nop 0\n\tv_writelane_b32 %0, %2, m0\n\tv_writelane_b32 %1, %3, m0"
                 : "+v"(lo), "+v"(hi) : "s"((u32)val), "s"((u32)(val >> 32)), "s"(lane) : "m0");
    v = ((u64)hi << 32) | lo;
}
#pragma clang diagnostic pop
__device__ __forceinline__ i64 wave_max_i64(i64 v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const i64 o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ i64 wave_scan_incl(i64 v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const i64 o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    return v;
}

template <int NR>
__device__ __forceinline__ int mask_lowest(const u64 (&m)[NR]) {
    if constexpr (NR == 2) return m[0] ? __builtin_ctzll(m[0]) : 64 + __builtin_ctzll(m[1]);
    else return __builtin_ctzll(m[0]);
}
template <int NR>
__device__ __forceinline__ bool mask_any(const u64 (&m)[NR]) {
    if constexpr (NR == 2) return (m[0] | m[1]) != 0;
    else return m[0] != 0;
}
// the row mask of column d (wave-uniform) as uniform words
template <int NR>
__device__ __forceinline__ void column_mask(const u64 (&cm)[NR][NR], int d, u64 (&out)[NR]) {
    const int dl = d & 63;
#pragma unroll
    for (int w = 0; w < NR; ++w) {
        if constexpr (NR == 2) out[w] = (d >> 6) ? rdl64(cm[1][w], dl) : rdl64(cm[0][w], dl);
        else out[w] = rdl64(cm[0][w], dl);
    }
}

// Embedding (paper Section 4.4 "Adapting an arbitrary matrix to a valid form"): loads the
// per-lane matrix Q of matrix b into LDS (row stride RS >= S words), raises every line to L =
// the largest row/column sum by virtual bytes - first on the diagonal, then row deficits poured
// into column deficits in ascending order, which makes the virtual part of cell (a, d) the
// overlap of the prefix-sum intervals [PR[a], ER[a]) and [PC[d], EC[d]) plus diag[a] on the
// diagonal - and leaves R = Q + A in LDS, bit 63 set where a cell holds virtual bytes.  PR, ER,
// diag stay in registers (per row of the lane), PC, EC go to LDS.  qmax receives the largest
// entry of Q (no cell ever holds more real bytes than that).
// PAIRS: when L < 2^31 a cell is left as two 32-bit halves instead - low: the residual Q + A,
// high: the real bytes Q - without a flag, so that whoever matches the cell reads both counts
// at once and never has to recompute the overlap.
// Common factor: when L does not fit 31 bits but every entry of Q is a multiple of 2^sh and
// L / 2^sh does, the whole matrix is divided by 2^sh (sh is returned; 0 otherwise).  Sums,
// deficits and virtual bytes are multiples of 2^sh as well, the decomposition of the divided
// matrix is the decomposition of the original with every byte count divided by 2^sh, so the
// caller runs on 32-bit words and shifts the byte counts it emits back.  Traffic built from
// whole tokens is of that kind: every entry a multiple of the token size.
// Returns -1 if kernel 1 flagged the matrix as invalid, else L (0: nothing to send), divided
// by 2^sh like everything else.
template <int NR, bool PAIRS = false>
__device__ __forceinline__ i64 embed_into_lds(const i64* __restrict__ wsQ,
                                              const i64* __restrict__ wsPart, int b, int S, int RS,
                                              int lane, u64* R, i64* PC, i64* EC,
                                              i64 (&diag)[NR], i64 (&PR)[NR], i64 (&ER)[NR],
                                              i64& qmax, int& sh) {
    sh = 0;
    {
        int bad = 0;
        for (int a = lane; a < S; a += 64) bad |= (int)wsPart[((size_t)b * S + a) * K1_PART + 2];
        if (ballot(bad != 0)) return -1;
    }
    const i64* Qg = wsQ + (size_t)b * S * S;
    u64 bits = 0;       // OR of the lane's entries: its trailing zeros are common to all of them
    if (RS == S) {
        for (int e = lane; e < S * S; e += 64) {
            const u64 v = (u64)Qg[e];
            R[e] = v;
            bits |= v;
        }
    } else {
        for (int e = lane; e < S * S; e += 64) {
            const int a = e / S;
            const u64 v = (u64)Qg[e];
            R[a * RS + (e - a * S)] = v;
            bits |= v;
        }
    }
    wave_sync();

    i64 rsum[NR], csum[NR];
    i64 cellmax = 0;
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int x = lane + 64 * k;
        rsum[k] = 0;
        csum[k] = 0;
        if (x < S) {
            for (int j = 0; j < S; ++j) {
                int d = j + x;
                d = d >= S ? d - S : d;
                const i64 v = (i64)R[x * RS + d];
                rsum[k] += v;
                cellmax = max(cellmax, v);
                csum[k] += (i64)R[j * RS + x];
            }
        }
    }
    qmax = (i64)uniform64((u64)wave_max_i64(cellmax));
    i64 lmax = 0;
#pragma unroll
    for (int k = 0; k < NR; ++k) lmax = max(lmax, max(rsum[k], csum[k]));
    i64 L = (i64)uniform64((u64)wave_max_i64(lmax));
    if (L == 0) return 0;
    if (L >= ((i64)1 << 31)) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) bits |= (u64)__shfl_xor((i64)bits, off, 64);
        const int tz = __builtin_ctzll(uniform64(bits));        // bits != 0 because L > 0
        if (tz > 0 && (L >> tz) < ((i64)1 << 31)) {
            sh = tz;
            for (int e = lane; e < S * RS; e += 64) R[e] >>= tz;     // pad words of a row included
            L >>= tz;
            qmax >>= tz;
#pragma unroll
            for (int k = 0; k < NR; ++k) { rsum[k] >>= tz; csum[k] >>= tz; }
            wave_sync();
        }
    }

    {
        i64 dr[NR], dc[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int x = lane + 64 * k;
            dr[k] = x < S ? L - rsum[k] : 0;
            dc[k] = x < S ? L - csum[k] : 0;
            diag[k] = min(dr[k], dc[k]);
            dr[k] -= diag[k];
            dc[k] -= diag[k];
        }
        i64 base_r = 0, base_c = 0;
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int x = lane + 64 * k;
            const i64 ir = wave_scan_incl(dr[k], lane);
            const i64 ic = wave_scan_incl(dc[k], lane);
            PR[k] = base_r + ir - dr[k];
            ER[k] = base_r + ir;
            if (x < S) {
                PC[x] = base_c + ic - dc[k];
                EC[x] = base_c + ic;
            }
            base_r += __shfl(ir, 63, 64);
            base_c += __shfl(ic, 63, 64);
        }
    }
    // PAIRS and L < 2^31: every word becomes {low half: residual, high half: real bytes}; the
    // virtual bytes are added to the low half only (the sum stays below 2^31: no carry) and no
    // flag is set
    const bool pairs = PAIRS && L < ((i64)1 << 31);
    const u64 vflag = pairs ? 0ull : VFLAG;
    if (pairs)
        for (int e = lane; e < S * RS; e += 64) R[e] |= R[e] << 32;
    wave_sync();
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int x = lane + 64 * k;
        if (x < S) {
            if (diag[k] > 0) R[x * RS + x] = (R[x * RS + x] + (u64)diag[k]) | vflag;
            if (ER[k] > PR[k]) {
                for (int j = 0; j < S; ++j) {
                    int d = j + x;
                    d = d >= S ? d - S : d;
                    const i64 l = max(PR[k], PC[d]);
                    const i64 h = min(ER[k], EC[d]);
                    if (h > l) R[x * RS + d] = (R[x * RS + d] + (u64)(h - l)) | vflag;
                }
            }
        }
    }
    wave_sync();
    return L;
}

// No residual exceeds L, the largest line sum: when L < 2^31 the n 64-bit words of R are
// repacked in place to 32-bit words (the flag in bit 63 is dropped).
__device__ __forceinline__ void repack_narrow(u64* R, int n, int lane) {
    u32* R32 = reinterpret_cast<u32*>(R);
    for (int e0 = 0; e0 < n; e0 += 64) {
        const int e = e0 + lane;
        u64 v = 0;
        if (e < n) v = R[e];
        wave_sync();                    // chunk read before its (lower) words are rewritten
        if (e < n) R32[e] = (u32)v;
    }
    wave_sync();
}

// Canonical augmenting search from the unmatched row r0 (wave-uniform) on the graph given by
// the column masks cm (bit a of cm[k][a / 64] set while cell (a, column lane + 64k) is an
// edge): level-synchronous, the lowest-numbered frontier row becomes the parent of a newly
// reached column, the search stops at the first level that reaches an unmatched column and
// takes the lowest-numbered one.  Frontiers, visited set and the unmatched columns FREEC are
// wave-uniform masks; the frontiers of levels >= 2 are parked in Fh (LDS, [level][2]) and the
// parents are recomputed while the path is flipped.  Updates mr (row -> column, -1 =
// unmatched) and FREEC; false if no augmenting path exists.
template <int NR>
__device__ __forceinline__ bool bfs_augment(int r0, const u64 (&cm)[NR][NR], int (&mr)[NR],
                                            u64 (&FREEC)[NR], u64* Fh, int S, int lane) {
    auto col_mask = [&](int d, u64 (&out)[NR]) { column_mask<NR>(cm, d, out); };
    auto lowest = [&](const u64 (&m)[NR]) -> int { return mask_lowest<NR>(m); };
    auto any = [&](const u64 (&m)[NR]) -> bool { return mask_any<NR>(m); };
        u64 F[NR], VIS[NR];
#pragma unroll
        for (int w = 0; w < NR; ++w) {
            F[w] = (r0 >> 6) == w ? 1ull << (r0 & 63) : 0;
            VIS[w] = 0;
        }
        int nfree = 0;
#pragma unroll
        for (int w = 0; w < NR; ++w) nfree += __builtin_popcountll(FREEC[w]);
        const bool few = nfree <= 2;
        int level = 1, dstar = -1, a = -1;
        for (;;) {
            if (few) {
                // few unmatched columns: test each against the frontier with scalar work
                u64 fr[NR];
#pragma unroll
                for (int w = 0; w < NR; ++w) fr[w] = FREEC[w];
                while (any(fr)) {
                    const int f = lowest(fr);
                    u64 cmf[NR];
                    col_mask(f, cmf);
#pragma unroll
                    for (int w = 0; w < NR; ++w) cmf[w] &= F[w];
                    if (any(cmf)) {
                        dstar = f;
                        a = lowest(cmf);
                        break;
                    }
#pragma unroll
                    for (int w = 0; w < NR; ++w)
                        if ((f >> 6) == w) fr[w] &= ~(1ull << (f & 63));
                }
                if (dstar >= 0) break;
            }
            u64 N[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                u64 cand = 0;
#pragma unroll
                for (int w = 0; w < NR; ++w) cand |= cm[k][w] & F[w];
                N[k] = ballot(cand != 0) & ~VIS[k];
            }
            if (!few) {
                u64 fr[NR];
#pragma unroll
                for (int w = 0; w < NR; ++w) fr[w] = N[w] & FREEC[w];
                if (any(fr)) {
                    dstar = lowest(fr);
                    u64 cmf[NR];
                    col_mask(dstar, cmf);
#pragma unroll
                    for (int w = 0; w < NR; ++w) cmf[w] &= F[w];
                    a = lowest(cmf);
                    break;
                }
            }
            if (!any(N)) return false;
#pragma unroll
            for (int w = 0; w < NR; ++w) VIS[w] |= N[w];
            if (level >= 2 && lane == 0) {
#pragma unroll
                for (int w = 0; w < NR; ++w) Fh[level * 2 + w] = F[w];
            }
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const int m = mr[k];
                u64 word;
                if constexpr (NR == 2) word = m < 64 ? N[0] : N[1];
                else word = N[0];
                F[k] = ballot(m >= 0 && ((word >> (m & 63)) & 1));
            }
            ++level;
        }
        // flip the path: column dstar <- row a <- its old column <- ... <- r0
        int d = dstar;
        for (int hops = 0;; ++hops) {
            if (hops > S) return false;
            int prev;
            if constexpr (NR == 2) prev = (a >> 6) ? (int)rdl(mr[1], a & 63) : (int)rdl(mr[0], a & 63);
            else prev = (int)rdl(mr[0], a & 63);
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                mr[k] = (lane + 64 * k == a) ? d : mr[k];
            }
            if (a == r0) break;
            d = prev;
            --level;
            u64 Fl[NR];
            if (level == 1) {
#pragma unroll
                for (int w = 0; w < NR; ++w) Fl[w] = (r0 >> 6) == w ? 1ull << (r0 & 63) : 0;
            } else {
#pragma unroll
                for (int w = 0; w < NR; ++w) {
                    const u64 x = Fh[level * 2 + w];
                    Fl[w] = ((u64)(u32)__builtin_amdgcn_readfirstlane((u32)(x >> 32)) << 32) |
                            (u64)(u32)__builtin_amdgcn_readfirstlane((u32)x);
                }
            }
            u64 cmd[NR];
            col_mask(d, cmd);
#pragma unroll
            for (int w = 0; w < NR; ++w) cmd[w] &= Fl[w];
            a = lowest(cmd);
        }
#pragma unroll
        for (int w = 0; w < NR; ++w)
            if ((dstar >> 6) == w) FREEC[w] &= ~(1ull << (dstar & 63));
        return true;
}

}  // namespace fastk
