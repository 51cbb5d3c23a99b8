// Kernel 2: embedding and Birkhoff decomposition of the server-level matrix.
//
// One wavefront (64 lanes) per traffic matrix.  The stage loop of Birkhoff's
// decomposition (paper Section 4.4 "Birkhoff's decomposition: overview") is a
// chain of dependent steps - find a perfect matching, take the smallest matched
// entry as the stage weight, subtract, repair the matching - so the design goal is
// the shortest possible dependent path per stage, not memory throughput:
//   * a single wavefront owns the matrix, so no step needs a workgroup barrier;
//     lane l owns rows l, l+64 and columns l, l+64 (S <= 128);
//   * the residual matrix R = Q + A lives in LDS (S*S int64) and is only touched
//     when the matching changes: the residual of each row's matched cell is held
//     in a register and written back when the row is re-matched;
//   * the support of R is kept as one S-bit row mask per column in registers, so a
//     breadth-first level of the augmenting-path search is two AND/compare
//     operations per lane plus wave ballots; the frontier is a wave-uniform mask;
//   * the virtual matrix A of the embedding (Section 4.4 "Adapting an arbitrary
//     matrix to a valid form") is never stored: pouring row deficits into column
//     deficits in ascending order makes A[a][d] the overlap of two prefix-sum
//     intervals (plus the diagonal term), recomputed when a cell gets matched.
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

#include "k1_rebalance.hpp"

namespace fastk {

constexpr int K2_THREADS = 64;

inline size_t k2_lds_bytes(int S) {
    return (size_t)S * S * sizeof(i64) + (size_t)2 * S * sizeof(i64);
}

__device__ __forceinline__ int rdlane(int v, int lane) {
    return __builtin_amdgcn_readlane(v, lane);
}

__device__ __forceinline__ u64 wave_min_u64(u64 v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const u64 o = __shfl_xor(v, off, 64);
        v = o < v ? o : v;
    }
    return v;
}

__device__ __forceinline__ i64 wave_max_i64(i64 v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const i64 o = __shfl_xor(v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ i64 wave_scan_incl(i64 v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const i64 o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    return v;
}

// NR = rows (and columns) per lane: 1 for S <= 64, 2 for S <= 128.
template <int NR>
__global__ void __launch_bounds__(K2_THREADS)
k2_birkhoff(const i64* __restrict__ wsQ, const i64* __restrict__ wsPart,
            int32_t* __restrict__ out_stages, i64* __restrict__ out_bytes,
            int32_t* __restrict__ out_num, i64* __restrict__ wsC, int S, int max_stages) {
    extern __shared__ __align__(16) unsigned char k2_smem[];
    i64* R = reinterpret_cast<i64*>(k2_smem);     // [S][S]
    i64* PC = R + (size_t)S * S;                  // [S] start of column d's deficit interval
    i64* EC = PC + S;                             // [S] end of it
    const int b = blockIdx.x;
    const int lane = threadIdx.x;

    // a negative entry anywhere in the matrix: no plan
    {
        int bad = 0;
        for (int a = lane; a < S; a += 64) bad |= (int)wsPart[((size_t)b * S + a) * K1_PART + 2];
        if (__ballot(bad != 0)) {
            if (lane == 0) out_num[b] = -1;
            return;
        }
    }

    // ---- load Q (per-lane bytes of every server pair, diagonal zero)
    const i64* Qg = wsQ + (size_t)b * S * S;
    for (int e = lane; e < S * S; e += 64) R[e] = Qg[e];
    __syncthreads();

    // ---- row / column sums, L = heaviest line (Section 4.4)
    i64 rsum[NR], csum[NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int x = lane + 64 * k;
        rsum[k] = 0;
        csum[k] = 0;
        if (x < S) {
            for (int j = 0; j < S; ++j) {
                int d = j + x;                     // rotated so that lanes hit different banks
                d = d >= S ? d - S : d;
                rsum[k] += R[(size_t)x * S + d];
                csum[k] += R[(size_t)j * S + x];
            }
        }
    }
    i64 lmax = 0;
#pragma unroll
    for (int k = 0; k < NR; ++k) lmax = max(lmax, max(rsum[k], csum[k]));
    const i64 L = wave_max_i64(lmax);
    if (L == 0) {
        if (lane == 0) out_num[b] = 0;
        return;
    }

    // ---- embedding: diagonal first, then row deficits poured into column deficits
    i64 diag[NR], PR[NR], ER[NR];
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
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int x = lane + 64 * k;
        if (x < S) {
            if (diag[k] > 0) R[(size_t)x * S + x] += diag[k];
            if (ER[k] > PR[k]) {
                for (int j = 0; j < S; ++j) {
                    int d = j + x;
                    d = d >= S ? d - S : d;
                    const i64 l = max(PR[k], PC[d]);
                    const i64 h = min(ER[k], EC[d]);
                    if (h > l) R[(size_t)x * S + d] += h - l;
                }
            }
        }
    }
    __syncthreads();

    // ---- support masks: bit a of cm[k] is set while R[a][column] > 0
    u64 cmLo[NR], cmHi[NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const int x = lane + 64 * k;
        cmLo[k] = 0;
        cmHi[k] = 0;
        if (x < S) {
            for (int a = 0; a < S; ++a) {
                const bool pos = R[(size_t)a * S + x] > 0;
                if (a < 64) cmLo[k] |= (u64)pos << a;
                else cmHi[k] |= (u64)pos << (a - 64);
            }
        }
    }

    int mr[NR], mc[NR], loaded[NR], par[NR];
    i64 rv[NR], av[NR];
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        mr[k] = -1;
        mc[k] = -1;
        loaded[k] = -1;
        par[k] = 0;
        rv[k] = 0;
        av[k] = 0;
    }

    // select / update slot `s` (wave-uniform) of a per-lane pair
    auto sel = [&](const int (&v)[NR], int s) -> int {
        if constexpr (NR == 2) return s ? v[1] : v[0];
        else return v[0];
    };

    // Augmenting path from unmatched row r0 (wave-uniform).  Returns false if none.
    auto augment = [&](int r0) -> bool {
        u64 Flo = r0 < 64 ? 1ull << r0 : 0;
        u64 Fhi = r0 >= 64 ? 1ull << (r0 - 64) : 0;
        bool vis[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) vis[k] = false;
        int dstar = -1;
        for (;;) {
            bool isnew[NR], isfree[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const u64 cl = cmLo[k] & Flo;
                const u64 ch = NR == 2 ? (cmHi[k] & Fhi) : 0;
                isnew[k] = !vis[k] && ((cl | ch) != 0);
                if (isnew[k]) {
                    par[k] = cl ? __builtin_ctzll(cl) : 64 + __builtin_ctzll(ch);
                    vis[k] = true;
                }
                isfree[k] = isnew[k] && mc[k] < 0;
            }
            const u64 f0 = __ballot(isfree[0]);
            const u64 f1 = NR == 2 ? __ballot(isfree[NR - 1]) : 0;
            if (f0 | f1) {
                dstar = f0 ? __builtin_ctzll(f0) : 64 + __builtin_ctzll(f1);
                break;
            }
            const u64 n0 = __ballot(isnew[0]);
            const u64 n1 = NR == 2 ? __ballot(isnew[NR - 1]) : 0;
            if ((n0 | n1) == 0) return false;
            // next frontier: the rows matched to the newly reached columns
            bool inF[NR];
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                const int m = mr[k];
                inF[k] = m >= 0 && (((m < 64 ? n0 : n1) >> (m & 63)) & 1);
            }
            Flo = __ballot(inF[0]);
            Fhi = NR == 2 ? __ballot(inF[NR - 1]) : 0;
        }
        // flip the path back to r0
        int d = dstar;
        for (int hops = 0;; ++hops) {
            if (hops > S) return false;            // cannot happen: a path visits each row once
            const int a = rdlane(sel(par, d >> 6), d & 63);
            const int prev = rdlane(sel(mr, a >> 6), a & 63);
#pragma unroll
            for (int k = 0; k < NR; ++k) {
                if (lane + 64 * k == a) mr[k] = d;
                if (lane + 64 * k == d) mc[k] = a;
            }
            if (a == r0) break;
            d = prev;
        }
        return true;
    };

    // Make rv / av describe the cell each row is matched to now.
    auto sync_matched = [&]() {
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int a = lane + 64 * k;
            if (a < S && mr[k] != loaded[k]) {
                if (loaded[k] >= 0 && rv[k] > 0) R[(size_t)a * S + loaded[k]] = rv[k];
                const int d = mr[k];
                rv[k] = R[(size_t)a * S + d];
                const i64 l = max(PR[k], PC[d]);
                const i64 h = min(ER[k], EC[d]);
                av[k] = (h > l ? h - l : 0) + (d == a ? diag[k] : 0);
                loaded[k] = d;
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
    sync_matched();

    // ---- stage loop
    const size_t obase = (size_t)b * max_stages;
    i64 Lrem = L;
    int s = 0;
    for (;;) {
        if (s >= max_stages) { status = -2; break; }
        u64 mine = ~0ull;
#pragma unroll
        for (int k = 0; k < NR; ++k)
            if (lane + 64 * k < S) mine = min(mine, (u64)rv[k]);
        const i64 c = (i64)wave_min_u64(mine);
        bool zero[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int a = lane + 64 * k;
            zero[k] = false;
            if (a < S) {
                const i64 realleft = rv[k] > av[k] ? rv[k] - av[k] : 0;
                const i64 real = min(c, realleft);
                out_stages[(obase + s) * S + a] = real > 0 ? mr[k] : -1;
                out_bytes[(obase + s) * S + a] = real;
                rv[k] -= c;
                zero[k] = rv[k] == 0;
            }
        }
        if (lane == 0) wsC[obase + s] = c;
        ++s;
        Lrem -= c;
        if (Lrem == 0) break;

        const u64 z0 = __ballot(zero[0]);
        const u64 z1 = NR == 2 ? __ballot(zero[NR - 1]) : 0;
        // unmatch every exhausted cell: column side drops the row from its support
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            const int m = mc[k];
            if (m >= 0 && (((m < 64 ? z0 : z1) >> (m & 63)) & 1)) {
                if (m < 64) cmLo[k] &= ~(1ull << m);
                else cmHi[k] &= ~(1ull << (m - 64));
                mc[k] = -1;
            }
            if (zero[k]) mr[k] = -1;
        }
        bool ok = true;
        for (u64 z = z0; z && ok; z &= z - 1) ok = augment(__builtin_ctzll(z));
        if (NR == 2)
            for (u64 z = z1; z && ok; z &= z - 1) ok = augment(64 + __builtin_ctzll(z));
        if (!ok) { status = -3; break; }
        sync_matched();
    }
    if (lane == 0) out_num[b] = status < 0 ? status : s;
}

}  // namespace fastk
