// Per-stage redistribution (paper Section 4.1 "Redistribution", Section 4.2 Step 3):
// after a stage's scale-out transfer, lane k of destination server d holds bytes
// that belong to other GPUs of d and forwards them over scale-up.
//
// Which bytes those are follows from a byte-identity policy (the paper fixes none):
//  * GPU (a,i)'s bytes for server d form one region ordered by destination GPU;
//  * balancing: the GPU keeps the head of the region and hands off the tail, cut
//    into the pieces X[i][k] of the lane-routing tile in ascending receiver k;
//  * lane k's send queue is its own head followed by the pieces handed in, in
//    ascending donor index;
//  * every stage in which a sends to d takes the next stage_bytes[s][a] bytes of
//    every lane's queue.
// With the traffic tile and the lane-routing tile X of the pair, every piece has a
// closed-form place: piece (i -> k) starts in lane k's queue at
//   qs = X[k][k] + sum_{i' < i, i' != k} X[i'][k]          (0 for the own head, i == k)
// and in row i's region at
//   u0 = X[i][i] + sum_{k' < k, k' != i} X[i][k']          (0 for the own head),
// and row i's bytes for GPU (d,j) sit in the region at [C_i(j), C_i(j+1)), C_i the
// prefix sums of the traffic tile's row i.  So the bytes of lane k's queue that come
// from row i and belong to (d,j) are the queue interval
//   [qs + clamp(C_i(j) - u0, 0, X[i][k]), qs + clamp(C_i(j+1) - u0, 0, X[i][k]))
// and a stage's G x G redistribution matrix is, per cell (k, j), the overlap of the
// stage's chunk [offset, offset + bytes) with those (at most G) intervals.
//
// rd_offsets   one thread per source server walks the stages in execution order
//              keeping the bytes already sent to every destination in LDS: the
//              per-stage send offsets; optionally also files every (stage, source)
//              under its server pair (count, scan, fill - all in LDS), so that
// rd_volumes   one wavefront per server pair builds the pair's 8 x 8 x 8 intervals
//              once (lane (k, j) keeps its 8 in registers) and then runs through
//              the pair's stages: overlap, row and column sums without the diagonal
//              by DPP, wave maximum, atomic max into the stage's scale-up volume;
// rd_matrices  one wavefront per (selected stage, source server) writes the whole
//              G x G matrix.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"

namespace fastk {

constexpr int RD_ROWS = 64;     // source servers per workgroup of rd_offsets (one wavefront)
constexpr int RD_UNROLL = 16;   // stages per batch of the pipelined walk

inline size_t rd_offsets_lds_bytes(int S, bool lists) {
    return (size_t)RD_ROWS * S * (lists ? sizeof(i64) + sizeof(int32_t) : sizeof(i64));
}

__global__ void __launch_bounds__(256) rd_zero(u64* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// grid (ceil(S / RD_ROWS), B), RD_ROWS threads.  Lane l owns source server a and the
// LDS column [*][l]; no two lanes share a word, so the kernel needs no barrier.
// The walk over the stages is a chain of dependent steps (stage index -> the stage's
// row -> the running offset in LDS), so it is software-pipelined by hand: while batch n
// of RD_UNROLL stages is processed, the rows of batch n+1 and the indices of batch n+2
// are in flight.
// ALL: S is a multiple of RD_ROWS, every lane owns a real source server (no store predicate).
// The pair lists have max_stages + 1 slots per source server: slot max_stages is a dump for the
// lanes that do not send in a stage, so that the list store needs no predicate either.
template <bool LISTS, bool ORDERED, bool ALL>
__global__ void __launch_bounds__(RD_ROWS)
rd_offsets(const int32_t* __restrict__ stages, const i64* __restrict__ stage_bytes,
           const int32_t* __restrict__ num_stages, const int32_t* __restrict__ order,
           i64* __restrict__ out_offset, int32_t* __restrict__ lstart, int32_t* __restrict__ lcnt,
           i64x2* __restrict__ list, int S, int max_stages) {
    extern __shared__ __align__(16) unsigned char rd_smem[];
    constexpr int U = RD_UNROLL;
    const int b = blockIdx.y;
    const int lane = threadIdx.x;
    const int a = blockIdx.x * RD_ROWS + lane;
    const int K = min(num_stages[b], max_stages);     // a count beyond the capacity is not trusted
    if (K <= 0) return;
    i64* sent = reinterpret_cast<i64*>(rd_smem);                    // [d][lane]
    int32_t* next = reinterpret_cast<int32_t*>(sent + (size_t)RD_ROWS * S);   // [d][lane]
    const bool live = ALL || a < S;
    const int ac = live ? a : S - 1;                                // clamped: loads stay in range
    for (int d = 0; d < S; ++d) {
        sent[d * RD_ROWS + lane] = 0;
        if constexpr (LISTS) next[d * RD_ROWS + lane] = 0;
    }
    const int32_t* st = stages + (size_t)b * max_stages * S;
    const i64* by = stage_bytes + (size_t)b * max_stages * S;
    const int32_t* ord = ORDERED ? order + (size_t)b * max_stages : nullptr;
    i64* off_out = out_offset + (size_t)b * max_stages * S;

    if constexpr (LISTS) {
        // how often does a send to each d, then where does each pair's list start
        for (int s0 = 0; s0 < K; s0 += 2 * U) {
            int dd[2 * U];
#pragma unroll
            for (int u = 0; u < 2 * U; ++u)
                dd[u] = s0 + u < K ? st[(size_t)(s0 + u) * S + ac] : -1;
#pragma unroll
            for (int u = 0; u < 2 * U; ++u)
                if (dd[u] >= 0 && dd[u] < S) atomicAdd(&next[dd[u] * RD_ROWS + lane], 1);
        }
        if (live) {
            int acc = 0;
            for (int d = 0; d < S; ++d) {
                const int c = next[d * RD_ROWS + lane];
                lstart[((size_t)b * S + a) * S + d] = acc;
                lcnt[((size_t)b * S + a) * S + d] = c;
                next[d * RD_ROWS + lane] = acc;
                acc += c;
            }
        }
    }

    const size_t lbase = ((size_t)b * S + ac) * (size_t)(max_stages + 1);
    // one stage: running offset of the pair (a, d) in LDS, optional list entry, send offset out.
    // Branch-free for an idle row (d < 0): it adds 0 to word 0 of the lane's column.  Lanes
    // beyond S work on a copy of row S-1 in their own LDS column and store nothing.
    auto stage = [&](int s, int d, i64 len) {
        const bool sends = d >= 0 && d < S;
        const int w = (sends ? d : 0) * RD_ROWS + lane;
        const i64 before = (i64)atomicAdd(reinterpret_cast<u64*>(&sent[w]), (u64)(sends ? len : 0));
        const i64 off = sends ? before : 0;
        if constexpr (LISTS) {
            const int pos = atomicAdd(&next[w], sends ? 1 : 0);
            if (live && sends && pos < max_stages) {    // pos < max_stages for any permutation
                i64x2 entry;
                entry.x = len;
                entry.y = s;
                list[lbase + pos] = entry;
            }
        }
        if (live) off_out[(size_t)s * S + a] = off;
    };
    // Stage indices of the batch at position e0: lane u holds the u-th (one coalesced load),
    // v_readlane hands them out as scalars.  An entry that is no stage index is clamped.
    auto load_idx = [&](int e0) -> int {
        if constexpr (ORDERED) return ord[e0 + (lane & (U - 1))];
        return e0 + (lane & (U - 1));
    };
    auto stage_of = [&](int iv, int u) -> int {
        const int s = __builtin_amdgcn_readlane(iv, u);
        return s < 0 ? 0 : (s >= K ? K - 1 : s);
    };
    auto load_rows = [&](int iv, int (&ss)[U], int (&dd)[U], i64 (&ln)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ss[u] = stage_of(iv, u);
            dd[u] = st[(size_t)ss[u] * S + ac];
            ln[u] = by[(size_t)ss[u] * S + ac];
        }
    };
    // A batch: first all fetch-and-adds (they queue up in the LDS pipe in program order, one
    // wait for the lot), then all stores.
    auto process = [&](const int (&ss)[U], const int (&dd)[U], const i64 (&ln)[U]) {
        i64 off[U];
        int pos[U];
        bool sends[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            sends[u] = dd[u] >= 0 && dd[u] < S;
            const int w = (sends[u] ? dd[u] : 0) * RD_ROWS + lane;
            off[u] = (i64)atomicAdd(reinterpret_cast<u64*>(&sent[w]), (u64)(sends[u] ? ln[u] : 0));
            if constexpr (LISTS) pos[u] = atomicAdd(&next[w], sends[u] ? 1 : 0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const i64 o = sends[u] ? off[u] : 0;
            if constexpr (LISTS) {
                i64x2 entry;                     // one 16-byte store: (bytes per lane, stage)
                entry.x = ln[u];
                entry.y = ss[u];
                // pos < max_stages for any permutation; everything else goes to the dump slot
                const int slot = sends[u] && pos[u] < max_stages ? pos[u] : max_stages;
                if (live) list[lbase + slot] = entry;
            }
            if (live) off_out[(size_t)ss[u] * S + a] = o;
        }
    };
    // Three batch buffers take the roles "being processed", "rows in flight", "indices in
    // flight" in turn, so no register is copied while its load is outstanding.
    const int nb = K / U;                       // full batches; the tail follows below
    int i0 = 0, i1 = 0, i2 = 0;
    int s0[U], s1[U], s2[U], d0[U], d1[U], d2[U];
    i64 l0[U], l1[U], l2[U];
    if (nb > 0) { i0 = load_idx(0); load_rows(i0, s0, d0, l0); }
    if (nb > 1) i1 = load_idx(U);
    for (int n = 0; n < nb; n += 3) {
        if (n + 1 < nb) load_rows(i1, s1, d1, l1);
        if (n + 2 < nb) i2 = load_idx((n + 2) * U);
        process(s0, d0, l0);
        if (n + 1 >= nb) break;
        if (n + 2 < nb) load_rows(i2, s2, d2, l2);
        if (n + 3 < nb) i0 = load_idx((n + 3) * U);
        process(s1, d1, l1);
        if (n + 2 >= nb) break;
        if (n + 3 < nb) load_rows(i0, s0, d0, l0);
        if (n + 4 < nb) i1 = load_idx((n + 4) * U);
        process(s2, d2, l2);
    }
    for (int e = nb * U; e < K; ++e) {
        int s = ORDERED ? ord[e] : e;
        s = s < 0 ? 0 : (s >= K ? K - 1 : s);
        stage(s, st[(size_t)s * S + ac], by[(size_t)s * S + ac]);
    }
}

// Wave-private LDS of the interval construction, in 8-byte words.
constexpr int RD_TILE_WORDS = 64 * 4 + 72;

// Builds, for lane (k, j) = (lane >> 3, lane & 7), the G queue intervals lo[i], hi[i]
// (i = source row) described at the top of this file, and returns the tile total.
// `t` is the wavefront's RD_TILE_WORDS words of LDS; every lane of the wavefront calls
// this together (the workgroup is one wavefront, so __syncthreads is a wave barrier).
__device__ __forceinline__ i64 rd_intervals(const i64* __restrict__ traffic_tile,
                                            const i64* __restrict__ x_tile, size_t row_stride,
                                            int G, i64* t, i64 lo[8], i64 hi[8]) {
    const int lane = threadIdx.x & 63;
    const int r = lane >> 3, c = lane & 7;
    const bool in = r < G && c < G;
    i64* TR = t;               // [i][j] traffic tile
    i64* XT = t + 64;          // [i][k] lane-routing tile
    i64* QS = t + 128;         // [i][k] start of piece (i -> k) in lane k's queue
    i64* U0 = t + 192;         // [i][k] start of piece (i -> k) in row i's region
    i64* CP = t + 256;         // [i][0..8] prefix sums of the traffic tile's row i
    const i64 tr = in ? traffic_tile[(size_t)r * row_stride + c] : 0;
    const i64 x = in ? x_tile[(size_t)r * row_stride + c] : 0;
    TR[lane] = tr;
    XT[lane] = x;
    __syncthreads();
    i64 cp = 0, qs = 0, u0 = 0;
    for (int m = 0; m < c; ++m) cp += TR[r * 8 + m];
    if (r != c) {
        qs = XT[c * 8 + c];
        for (int m = 0; m < r; ++m)
            if (m != c) qs += XT[m * 8 + c];
        u0 = XT[r * 8 + r];
        for (int m = 0; m < c; ++m)
            if (m != r) u0 += XT[r * 8 + m];
    }
    CP[r * 9 + c] = cp;
    if (c == 7) CP[r * 9 + 8] = cp + tr;
    QS[lane] = qs;
    U0[lane] = u0;
    __syncthreads();
    const int k = r, j = c;
    i64 total = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const i64 piece = XT[i * 8 + k];
        const i64 q0 = QS[i * 8 + k];
        const i64 r0 = U0[i * 8 + k];
        const i64 c0 = CP[i * 9 + j] - r0;
        const i64 c1 = CP[i * 9 + j + 1] - r0;
        lo[i] = q0 + min(max(c0, (i64)0), piece);
        hi[i] = q0 + min(max(c1, (i64)0), piece);
        total += CP[i * 9 + 8];
    }
    return total;
}

// Bytes of the chunk [off, end) that fall into the lane's intervals.
template <typename I>
__device__ __forceinline__ I rd_cell(const I lo[8], const I hi[8], I off, I end) {
    I m = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const I l = max(lo[i], off);
        const I h = min(hi[i], end);
        m += h > l ? h - l : (I)0;
    }
    return m;
}

__device__ __forceinline__ int dpp_sum8(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);    // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);   // row_half_mirror
    return v;
}
__device__ __forceinline__ i64 dpp_sum8(i64 v) {
    v += dpp_i64<0xB1>(v);
    v += dpp_i64<0x4E>(v);
    v += dpp_i64<0x141>(v);
    return v;
}
__device__ __forceinline__ int dpp_ror8(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false);   // row_ror:8
}
__device__ __forceinline__ i64 dpp_ror8(i64 v) { return dpp_i64<0x128>(v); }

// Exchange between the two 16-lane rows of each half (xor 16) and between the two halves
// (xor 32) with the gfx950 row-swap instructions: swap(v, v) returns the pair
// (rows 0,0,2,2 | rows 1,1,3,3) resp. (lower half twice | upper half twice), so one
// commutative operation on the pair leaves the reduction in every lane - no LDS round trip.
struct rd_sum { template <typename T> __device__ T operator()(T a, T b) const { return a + b; } };
struct rd_max { template <typename T> __device__ T operator()(T a, T b) const { return a > b ? a : b; } };
template <bool ROWS, typename OP>
__device__ __forceinline__ int rd_swap_reduce(int v, OP op) {
    if constexpr (ROWS) {
        const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        return op((int)r[0], (int)r[1]);
    } else {
        const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
        return op((int)r[0], (int)r[1]);
    }
}
template <bool ROWS, typename OP>
__device__ __forceinline__ i64 rd_swap_reduce(i64 v, OP op) {
    const unsigned lo = (unsigned)(u64)v, hi = (unsigned)((u64)v >> 32);
    i64 a, b;
    if constexpr (ROWS) {
        const auto l = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto h = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        a = (i64)(((u64)h[0] << 32) | l[0]);
        b = (i64)(((u64)h[1] << 32) | l[1]);
    } else {
        const auto l = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto h = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        a = (i64)(((u64)h[0] << 32) | l[0]);
        b = (i64)(((u64)h[1] << 32) | l[1]);
    }
    return op(a, b);
}
template <int CTRL> __device__ __forceinline__ int rd_dpp_get(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL> __device__ __forceinline__ i64 rd_dpp_get(i64 v) { return dpp_i64<CTRL>(v); }

// Largest, over the 8 GPUs, of max(bytes forwarded, bytes received): m is the lane's
// cell (k, j) of the redistribution matrix with the diagonal already zeroed.  The result is
// in every lane.
template <typename I>
__device__ __forceinline__ I rd_volume(I m) {
    const I fwd = dpp_sum8(m);                              // row k: what lane k forwards
    I recv = m + dpp_ror8(m);                               // column j: rows k and k ^ 1 ...
    recv = rd_swap_reduce<true>(recv, rd_sum());            // ... the other 16-lane row ...
    recv = rd_swap_reduce<false>(recv, rd_sum());           // ... and the other half
    I v = max(fwd, recv);
    v = max(v, rd_dpp_get<0xB1>(v));                        // quad_perm [1,0,3,2]
    v = max(v, rd_dpp_get<0x4E>(v));                        // quad_perm [2,3,0,1]
    v = max(v, rd_dpp_get<0x141>(v));                       // row_half_mirror
    v = max(v, rd_dpp_get<0x140>(v));                       // row_mirror
    v = rd_swap_reduce<true>(v, rd_max());
    v = rd_swap_reduce<false>(v, rd_max());
    return v;
}

// The pair's list is in execution order, so a stage's send offset is the running sum of the
// bytes of the entries before it.
template <typename I>
__device__ __forceinline__ void rd_run_pair(const i64 lo64[8], const i64 hi64[8], bool diag,
                                            const i64x2* __restrict__ list, int n,
                                            u64* __restrict__ redis) {
    I lo[8], hi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { lo[i] = (I)lo64[i]; hi[i] = (I)hi64[i]; }
    i64 off = 0;
    for (int e = 0; e < n; ++e) {
        const i64x2 entry = list[e];
        const int s = (int)entry.y;
        const i64 end = off + entry.x;
        I m = rd_cell<I>(lo, hi, (I)off, (I)end);
        off = end;
        if (diag) m = 0;
        const I v = rd_volume<I>(m);
        if ((threadIdx.x & 63) == 0 && v > 0) atomicMax(&redis[s], (u64)v);
    }
}

// grid (S * S, B), 64 threads: one wavefront per ordered server pair (a, d).
__global__ void __launch_bounds__(64)
rd_volumes(const i64* __restrict__ traffic, const i64* __restrict__ X,
           const int32_t* __restrict__ num_stages, const int32_t* __restrict__ lstart,
           const int32_t* __restrict__ lcnt, const i64x2* __restrict__ list,
           u64* __restrict__ redis, int S, int G, int max_stages) {
    __shared__ i64 t[RD_TILE_WORDS];
    const int b = blockIdx.y;
    const int a = blockIdx.x / S;
    const int d = blockIdx.x - a * S;
    if (a == d || num_stages[b] <= 0) return;
    const size_t pair = ((size_t)b * S + a) * S + d;
    const int n = lcnt[pair];
    if (n <= 0) return;
    const int N = S * G;
    const size_t tile = ((size_t)b * N + (size_t)a * G) * N + (size_t)d * G;
    i64 lo[8], hi[8];
    const i64 total = rd_intervals(traffic + tile, X + tile, (size_t)N, G, t, lo, hi);
    const size_t lbase = ((size_t)b * S + a) * (size_t)(max_stages + 1) + lstart[pair];
    const int lane = threadIdx.x & 63;
    const bool diag = (lane >> 3) == (lane & 7);
    u64* out = redis + (size_t)b * max_stages;
    if (total < ((i64)1 << 31))
        rd_run_pair<int>(lo, hi, diag, list + lbase, n, out);
    else
        rd_run_pair<i64>(lo, hi, diag, list + lbase, n, out);
}

// grid (S, n_sel), 64 threads: one wavefront per (selected stage, source server).
// sel[q] = (b, s); out[q][d][k][j], zero-filled beforehand.
__global__ void __launch_bounds__(64)
rd_matrices(const i64* __restrict__ traffic, const i64* __restrict__ X,
            const int32_t* __restrict__ stages, const i64* __restrict__ stage_bytes,
            const i64* __restrict__ stage_offset, const int32_t* __restrict__ num_stages,
            const int32_t* __restrict__ sel, i64* __restrict__ out, int B, int S, int G,
            int max_stages) {
    __shared__ i64 t[RD_TILE_WORDS];
    const int q = blockIdx.y;
    const int a = blockIdx.x;
    const int b = sel[2 * q];
    const int s = sel[2 * q + 1];
    if (b < 0 || b >= B) return;
    if (s < 0 || s >= min(num_stages[b], max_stages)) return;
    const size_t row = ((size_t)b * max_stages + s) * S + a;
    const int d = stages[row];
    if (d < 0 || d >= S || d == a) return;
    const int N = S * G;
    const size_t tile = ((size_t)b * N + (size_t)a * G) * N + (size_t)d * G;
    i64 lo[8], hi[8];
    (void)rd_intervals(traffic + tile, X + tile, (size_t)N, G, t, lo, hi);
    const i64 off = stage_offset[row];
    const i64 m = rd_cell<i64>(lo, hi, off, off + stage_bytes[row]);
    const int lane = threadIdx.x & 63;
    const int k = lane >> 3, j = lane & 7;
    if (k < G && j < G) out[(((size_t)q * S + d) * G + k) * G + j] = m;
}

}  // namespace fastk
