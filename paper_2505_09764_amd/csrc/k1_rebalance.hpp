// Kernel 1: server aggregation, sender balancing and collapse.
//
// One workgroup per (matrix b, source server a) handles the G x N row block of
// the traffic matrix that belongs to server a (64 KiB in, 64 KiB out at S = 128,
// G = 8, both contiguous):
//   phase A  reads the block once, 16 bytes per lane with consecutive lanes on
//            consecutive addresses, and reduces every cross-server tile row to its
//            row sum r_i(a,d) (paper Section 4.1 "Example setup": a tile's row
//            sums are what each GPU sends to that server).  The G/2 lanes that
//            share a tile row add their partial sums with DPP lane exchanges;
//   phase B  one thread per tile: tile total T[a][d], lane targets floor/ceil(T/G),
//            and in one ascending pass over the tile's rows each row's surplus or
//            deficit and where it starts among the tile's surpluses / deficits
//            (Section 4.1 "Mitigating sender skew"); the per-lane server entry
//            Q[a][d] = ceil(T/G) of the merged peer transfer (Section 4.1
//            "Mitigating receiver skew", Section 4.2 Fig. 6);
//   phase C  writes the lane-routing matrix X, again 16 bytes per lane.  Pouring
//            surpluses into deficits in ascending index order means surplus row i
//            covers the byte interval [PS_i, PS_i + s_i) and deficit row k the
//            interval [PD_k, PD_k + d_k) of the same line, so X[i][k] is the length
//            of their intersection - every output element is independent of the
//            others.  Two surplus rows (or two deficit rows) never intersect, so
//            only the sender's side needs the surplus test.
// The block also leaves, for the cost model, the largest per-GPU hand-off
// volume (balancing) and intra-server volume of its server.
//
// HBM traffic: the row block is read once (8*G*N bytes) and X written once
// (8*G*N bytes), both with the non-temporal hint since neither is touched again
// by this kernel; everything else lives in LDS (3 tables of S*G words).
//
// k1_block is the general form (any G up to 8, any alignment).  For G = 2, 4, 8 and 16-byte
// aligned buffers k1_block_tiles below computes the same outputs without the three phases:
// each tile is worked out in registers by the lanes that loaded it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fastk {

typedef long long i64;
typedef unsigned long long u64;
typedef long long ll2 __attribute__((ext_vector_type(2)));

struct alignas(16) i64x2 { i64 x, y; };

constexpr int K1_THREADS = 256;
constexpr int K1_MAX_S = 128;            // FAST_MAX_SERVERS: bounds the unrolled per-thread work
constexpr u64 K1_SURPLUS_BIT = 1ull << 63;
constexpr int K1_SLOTS = 8;              // partial sums per block-wide total (spreads LDS atomics)

// Per-block record left for kernels 2 and 3: [b][a][4]
//   0: max over the server's GPUs of max(bytes handed off, bytes handed in)
//   1: max over the server's GPUs of max(intra-server bytes out, in)
//   2: 1 if a negative off-diagonal entry was seen in the block
//   3: sum_d T[a][d]
constexpr int K1_PART = 4;

inline size_t k1_lds_bytes(int S, int G) {
    return (size_t)S * G * 3 * sizeof(i64) +
           (size_t)((2 * G + 1) * K1_SLOTS + 2 * G + 2) * sizeof(i64);
}

// 64-bit value of the lane selected by DPP control CTRL (every lane has a source).
template <int CTRL>
__device__ __forceinline__ i64 dpp_i64(i64 x) {
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(u64)x, CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)((u64)x >> 32), CTRL, 0xf, 0xf, false);
    return (i64)(((u64)(unsigned)hi << 32) | (unsigned)lo);
}

template <int G, bool VEC>
__device__ __forceinline__ void
k1_block(const i64* __restrict__ traffic, i64* __restrict__ X, i64* __restrict__ wsT,
         i64* __restrict__ wsQ, i64* __restrict__ wsPart, int S, int a, int b,
         unsigned char* k1_smem) {
    constexpr int EPL = VEC ? 2 : 1;         // elements per lane
    constexpr int LPR = G / EPL;             // lanes per tile row
    constexpr bool POW2 = (LPR & (LPR - 1)) == 0;
    constexpr int MAXIT = (K1_MAX_S * LPR + K1_THREADS - 1) / K1_THREADS;
    const int N = S * G;
    const int P = S * G;                     // tile rows of the block, index p = d*G + i
    const int rowl = S * LPR;                // lanes per GPU row
    u64* lo = reinterpret_cast<u64*>(k1_smem);
    i64* hi = reinterpret_cast<i64*>(lo + P);
    i64* kept = hi + P;                      // holds the tile row sums until phase B
    u64* acc = reinterpret_cast<u64*>(kept + P);   // [(2G+1)][SLOTS]
    i64* intra_in = reinterpret_cast<i64*>(acc + (2 * G + 1) * K1_SLOTS);
    i64* intra_out = intra_in + G;
    i64* misc = intra_out + G;               // [0] negative flag
    const int tid = threadIdx.x;

    for (int t = tid; t < (2 * G + 1) * K1_SLOTS + 2 * G + 2; t += K1_THREADS) acc[t] = 0;
    if constexpr (!POW2) {
        for (int t = tid; t < P; t += K1_THREADS) kept[t] = 0;
    }
    __syncthreads();

    const i64* blk = traffic + ((size_t)b * N + (size_t)a * G) * N;

    // ---- phase A: lane hp of GPU row i holds elements [hp*EPL, hp*EPL + EPL) of that row.
    // All loads of IB rows are issued before the first one is consumed.
    {
        i64 orv = 0;
        constexpr int IB = G >= 4 ? 4 : G;   // GPU rows whose loads are in flight together
#pragma unroll
        for (int i0 = 0; i0 < G; i0 += IB) {
            i64 w[IB][MAXIT][EPL];
#pragma unroll
            for (int ii = 0; ii < IB; ++ii) {
#pragma unroll
                for (int it = 0; it < MAXIT; ++it) {
                    const int hp = tid + it * K1_THREADS;
                    const i64* src = blk + (size_t)(i0 + ii) * N + (size_t)hp * EPL;
                    if constexpr (VEC) {
                        ll2 t = {0, 0};
                        if (i0 + ii < G && hp < rowl) t = __builtin_nontemporal_load(reinterpret_cast<const ll2*>(src));
                        w[ii][it][0] = t.x;
                        w[ii][it][1] = t.y;
                    } else {
                        w[ii][it][0] = (i0 + ii < G && hp < rowl) ? __builtin_nontemporal_load(src) : 0;
                    }
                }
            }
#pragma unroll
            for (int ii = 0; ii < IB; ++ii) {
                const int i = i0 + ii;
                if (i >= G) continue;
#pragma unroll
                for (int it = 0; it < MAXIT; ++it) {
                    const int hp = tid + it * K1_THREADS;
                    const int d = hp / LPR;
                    const int k = (hp - d * LPR) * EPL;
                    const bool live = hp < rowl;
                    i64 sum = 0;
                    if (live && d == a) {
#pragma unroll
                        for (int c = 0; c < EPL; ++c) {
                            i64 x = w[ii][it][c];
                            if (k + c == i) x = 0;      // the GPU diagonal uses no link
                            orv |= x;
                            sum += x;
                            if (x) atomicAdd(reinterpret_cast<u64*>(&intra_in[k + c]), (u64)x);
                        }
                        if (sum) atomicAdd(reinterpret_cast<u64*>(&intra_out[i]), (u64)sum);
                    } else {
#pragma unroll
                        for (int c = 0; c < EPL; ++c) { orv |= w[ii][it][c]; sum += w[ii][it][c]; }
                    }
                    if constexpr (POW2) {
                        if constexpr (LPR >= 2) sum += dpp_i64<0xB1>(sum);    // quad_perm [1,0,3,2]
                        if constexpr (LPR >= 4) sum += dpp_i64<0x4E>(sum);    // quad_perm [2,3,0,1]
                        if constexpr (LPR >= 8) sum += dpp_i64<0x141>(sum);   // row_half_mirror
                        if (live && k == 0) kept[d * G + i] = sum;
                    } else {
                        if (live) atomicAdd(reinterpret_cast<u64*>(&kept[d * G + i]), (u64)sum);
                    }
                }
            }
        }
        if (orv < 0) misc[0] = 1;
    }
    __syncthreads();

    // ---- phase B: one thread per tile (a, d); p = d*G + k indexes the tables
    for (int d = tid; d < S; d += K1_THREADS) {
        i64 tot = 0, Q = 0;
        if (d == a) {
#pragma unroll
            for (int k = 0; k < G; ++k) { lo[d * G + k] = 0; hi[d * G + k] = 0; kept[d * G + k] = 0; }
        } else {
            i64 rr[G];
#pragma unroll
            for (int k = 0; k < G; ++k) { rr[k] = kept[d * G + k]; tot += rr[k]; }
            const i64 q = tot / G;
            const int rho = (int)(tot - q * G);
            Q = q + (rho > 0 ? 1 : 0);
            i64 ps = 0, pd = 0;
            const int slot = d & (K1_SLOTS - 1);
#pragma unroll
            for (int k = 0; k < G; ++k) {
                const i64 tk = q + (k < rho ? 1 : 0);
                const i64 diff = rr[k] - tk;
                const bool surplus = diff > 0;
                const i64 sk = surplus ? diff : 0;
                const i64 dk = sk - diff;
                const i64 base = surplus ? ps : pd;
                lo[d * G + k] = (u64)base | (surplus ? K1_SURPLUS_BIT : 0ull);
                hi[d * G + k] = base + (surplus ? sk : dk);
                kept[d * G + k] = rr[k] - sk;
                ps += sk;
                pd += dk;
                atomicAdd(&acc[k * K1_SLOTS + slot], (u64)sk);
                atomicAdd(&acc[(G + k) * K1_SLOTS + slot], (u64)dk);
            }
            atomicAdd(&acc[2 * G * K1_SLOTS + slot], (u64)tot);
        }
        wsT[((size_t)b * S + a) * S + d] = tot;
        wsQ[((size_t)b * S + a) * S + d] = Q;
    }
    __syncthreads();

    if (tid >= K1_THREADS - 64) {
        // last wave: lane j < 2G sums GPU j's hand-off (or hand-in) slots, lane 2G the tile totals
        const int j = tid - (K1_THREADS - 64);
        u64 s = 0;
        if (j < 2 * G + 1) {
#pragma unroll
            for (int k = 0; k < K1_SLOTS; ++k) s += acc[j * K1_SLOTS + k];
        }
        i64 bal = j < 2 * G ? (i64)s : 0;
        i64 intra = j < 2 * G ? intra_in[j] : 0;      // intra_in and intra_out are adjacent
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {
            bal = max(bal, __shfl_xor(bal, m));
            intra = max(intra, __shfl_xor(intra, m));
        }
        i64* part = wsPart + ((size_t)b * S + a) * K1_PART;
        if (j == 0) { part[0] = bal; part[1] = intra; part[2] = misc[0]; }
        if (j == 2 * G) part[3] = (i64)s;
    }

    // ---- phase C: lane-routing matrix, same lane-to-element mapping as phase A
    i64* xblk = X + ((size_t)b * N + (size_t)a * G) * N;
#pragma unroll
    for (int i = 0; i < G; ++i) {
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) {
            const int hp = tid + it * K1_THREADS;
            if (hp >= rowl) continue;
            const int d = hp / LPR;
            const int k = (hp - d * LPR) * EPL;
            const int p = d * G + i;
            const u64 lo_i = lo[p];
            const i64 slo = (i64)(lo_i & ~K1_SURPLUS_BIT);
            const i64 shi = (lo_i & K1_SURPLUS_BIT) ? hi[p] : slo;   // a deficit row hands nothing off
            const i64 kept_i = kept[p];
            i64 out[EPL];
#pragma unroll
            for (int c = 0; c < EPL; ++c) {
                const i64 lk = (i64)(lo[d * G + k + c] & ~K1_SURPLUS_BIT);
                const i64 hk = hi[d * G + k + c];
                const i64 l = max(slo, lk);
                const i64 h = min(shi, hk);
                const i64 w = h - l;
                out[c] = (k + c == i) ? kept_i : (w > 0 ? w : 0);
            }
            i64* dst = xblk + (size_t)i * N + (size_t)hp * EPL;
            if constexpr (VEC) {
                ll2 t = {out[0], out[1]};
                __builtin_nontemporal_store(t, reinterpret_cast<ll2*>(dst));
            } else {
                __builtin_nontemporal_store(out[0], dst);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The same block without the load -> barrier -> store shape (G = 2, 4, 8 with 16-byte
// aligned buffers).  A tile's balancing depends on that tile's G row sums only, and the G/2
// lanes that load a tile's rows (two columns each) are neighbours: after the DPP exchange
// each of them holds all G row sums, works the tile out in registers - targets, surplus and
// deficit intervals, its own two columns of X - and stores its part of X right away, 16 bytes
// per lane on the addresses it loaded from.  No LDS tables, no barrier between the loads and
// the stores: a wavefront's stores overlap the other wavefronts' loads, as in a plain copy.
// Only the per-server records still go through LDS (the same partial-sum slots, one
// lane per tile adds to them), and the block needs two barriers in all.
// ---------------------------------------------------------------------------
inline size_t k1_tiles_lds_bytes(int G) {
    return (size_t)((2 * G + 1) * K1_SLOTS + 2 * G + 2) * sizeof(i64);
}

template <int G>
__device__ __forceinline__ void
k1_block_tiles(const i64* __restrict__ traffic, i64* __restrict__ X, i64* __restrict__ wsT,
               i64* __restrict__ wsQ, i64* __restrict__ wsPart, int S, int a, int b,
               unsigned char* k1_smem) {
    constexpr int LPR = G / 2;               // lanes per tile row (two elements per lane)
    static_assert(G % 2 == 0 && (LPR & (LPR - 1)) == 0 && LPR <= 4, "G = 2, 4 or 8");
    constexpr int MAXIT = (K1_MAX_S * LPR + K1_THREADS - 1) / K1_THREADS;
    const int N = S * G;
    const int rowl = S * LPR;                // lanes per GPU row
    u64* acc = reinterpret_cast<u64*>(k1_smem);            // [(2G+1)][SLOTS]
    i64* intra_in = reinterpret_cast<i64*>(acc + (2 * G + 1) * K1_SLOTS);
    i64* intra_out = intra_in + G;
    i64* misc = intra_out + G;               // [0] negative flag
    const int tid = threadIdx.x;
    for (int t = tid; t < (2 * G + 1) * K1_SLOTS + 2 * G + 2; t += K1_THREADS) acc[t] = 0;
    __syncthreads();

    const i64* blk = traffic + ((size_t)b * N + (size_t)a * G) * N;
    i64* xblk = X + ((size_t)b * N + (size_t)a * G) * N;
    const int ql = tid & (LPR - 1);          // which pair of columns of the tile this lane holds
    i64 orv = 0;
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
        const int hp = tid + it * K1_THREADS;
        if ((hp & ~63) >= rowl) break;       // nothing left for this wavefront (wave-uniform)
        const bool live = hp < rowl;
        const int d = hp / LPR;
        const bool intra = live && d == a;

        // the tile's rows: two columns per lane, all loads in flight together
        ll2 w[G];
#pragma unroll
        for (int i = 0; i < G; ++i) {
            w[i] = ll2{0, 0};
            if (live) w[i] = __builtin_nontemporal_load(reinterpret_cast<const ll2*>(blk + (size_t)i * N + (size_t)hp * 2));
        }
        i64 r[G];
        i64 col0 = 0, col1 = 0;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            i64 x0 = w[i].x, x1 = w[i].y;
            if (intra) {                     // the GPU diagonal uses no link
                if (2 * ql == i) x0 = 0;
                if (2 * ql + 1 == i) x1 = 0;
                col0 += x0;
                col1 += x1;
            }
            orv |= x0 | x1;
            i64 sum = x0 + x1;
            if constexpr (LPR >= 2) sum += dpp_i64<0xB1>(sum);    // quad_perm [1,0,3,2]
            if constexpr (LPR >= 4) sum += dpp_i64<0x4E>(sum);    // quad_perm [2,3,0,1]
            r[i] = sum;
        }
        if (intra) {
            // intra-server tile: per-GPU bytes out (row sums) and in (column sums); nothing to balance
            intra_in[2 * ql] = col0;
            intra_in[2 * ql + 1] = col1;
            if (ql == 0) {
#pragma unroll
                for (int i = 0; i < G; ++i) intra_out[i] = r[i];
            }
#pragma unroll
            for (int i = 0; i < G; ++i) r[i] = 0;
        }

        // the tile, worked out by each of its lanes - in 32-bit arithmetic when every tile of the
        // wavefront has non-negative row sums and a total below 2^31 (all intermediate values
        // are then bounded by the total), in 64-bit arithmetic otherwise
        i64 tot = 0, rneg = 0;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            tot += r[i];
            rneg |= r[i];
        }
        const bool book = live && ql == 0 && d != a;       // one lane per cross-server tile keeps the books
        const int slot = d & (K1_SLOTS - 1);
        auto tile = [&](auto tag) {
            typedef decltype(tag) V;
            V rv[G];
#pragma unroll
            for (int i = 0; i < G; ++i) rv[i] = (V)r[i];
            const V q = (V)tot / (V)G;
            const int rho = (int)((V)tot - q * (V)G);
            // first pass over the lanes k of the tile: where each surplus / deficit starts on its
            // line; this lane keeps the intervals of its own two columns, one lane keeps the books
            V lk[2] = {0, 0}, hk[2] = {0, 0};
            {
                V ps = 0, pd = 0;
#pragma unroll
                for (int k = 0; k < G; ++k) {
                    const V tk = q + (k < rho ? 1 : 0);
                    const V diff = rv[k] - tk;
                    const bool surplus = diff > 0;
                    const V sk = surplus ? diff : 0;
                    const V dk = sk - diff;
                    const V base = surplus ? ps : pd;
                    if ((k >> 1) == ql) {
                        lk[k & 1] = base;
                        hk[k & 1] = base + (surplus ? sk : dk);
                    }
                    ps += sk;
                    pd += dk;
                    if (book) {
                        atomicAdd(&acc[k * K1_SLOTS + slot], (u64)(i64)sk);
                        atomicAdd(&acc[(G + k) * K1_SLOTS + slot], (u64)(i64)dk);
                    }
                }
            }
            if (live && ql == 0) {
                wsT[((size_t)b * S + a) * S + d] = tot;
                wsQ[((size_t)b * S + a) * S + d] = (i64)(q + (rho > 0 ? 1 : 0));
            }
            // second pass over the rows i: row i hands off the interval [ps, ps + s_i) of the
            // surplus line (empty for a deficit row); this lane's two columns of row i go out at once
            if (live) {
                V ps = 0;
#pragma unroll
                for (int i = 0; i < G; ++i) {
                    const V ti = q + (i < rho ? 1 : 0);
                    const V diff = rv[i] - ti;
                    const V si = diff > 0 ? diff : 0;
                    V out[2];
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const V l = max(ps, lk[c]);
                        const V h = min((V)(ps + si), hk[c]);
                        const V wd = h - l;
                        out[c] = wd > 0 ? wd : 0;
                    }
                    if ((i >> 1) == ql) out[i & 1] = rv[i] - si;    // what the GPU keeps for its own lane
                    ps += si;
                    __builtin_nontemporal_store(ll2{(i64)out[0], (i64)out[1]},
                                                reinterpret_cast<ll2*>(xblk + (size_t)i * N + (size_t)hp * 2));
                }
            }
        };
        if (book) atomicAdd(&acc[2 * G * K1_SLOTS + slot], (u64)tot);
        const bool wide = __builtin_amdgcn_ballot_w64(rneg < 0 || tot >= ((i64)1 << 31)) != 0;
        if (wide) tile((i64)0);
        else tile((int)0);
    }
    if (orv < 0) misc[0] = 1;
    __syncthreads();

    if (tid >= K1_THREADS - 64) {
        // last wave: lane j < 2G sums GPU j's hand-off (or hand-in) slots, lane 2G the tile totals
        const int j = tid - (K1_THREADS - 64);
        u64 s = 0;
        if (j < 2 * G + 1) {
#pragma unroll
            for (int k = 0; k < K1_SLOTS; ++k) s += acc[j * K1_SLOTS + k];
        }
        i64 bal = j < 2 * G ? (i64)s : 0;
        i64 intra = j < 2 * G ? intra_in[j] : 0;      // intra_in and intra_out are adjacent
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {
            bal = max(bal, __shfl_xor(bal, m));
            intra = max(intra, __shfl_xor(intra, m));
        }
        i64* part = wsPart + ((size_t)b * S + a) * K1_PART;
        if (j == 0) { part[0] = bal; part[1] = intra; part[2] = misc[0]; }
        if (j == 2 * G) part[3] = (i64)s;
    }
}

template <int G>
__global__ void __launch_bounds__(K1_THREADS)
k1_rebalance_tiles(const i64* __restrict__ traffic, i64* __restrict__ X, i64* __restrict__ wsT,
                   i64* __restrict__ wsQ, i64* __restrict__ wsPart, int S) {
    extern __shared__ __align__(16) unsigned char k1_smem[];
    k1_block_tiles<G>(traffic, X, wsT, wsQ, wsPart, S, (int)blockIdx.x, (int)blockIdx.y, k1_smem);
}

// One workgroup per (source server blockIdx.x, matrix blockIdx.y).
template <int G, bool VEC>
__global__ void __launch_bounds__(K1_THREADS)
k1_rebalance(const i64* __restrict__ traffic, i64* __restrict__ X, i64* __restrict__ wsT,
             i64* __restrict__ wsQ, i64* __restrict__ wsPart, int S) {
    extern __shared__ __align__(16) unsigned char k1_smem[];
    k1_block<G, VEC>(traffic, X, wsT, wsQ, wsPart, S, (int)blockIdx.x, (int)blockIdx.y, k1_smem);
}

}  // namespace fastk
