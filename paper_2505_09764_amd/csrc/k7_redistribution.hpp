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
//              per-stage send offsets; the walk is cut into chunks that run side by side,
//              each starting from the totals of the chunks before it (rd_chunk_totals);
// rd_volumes   one workgroup per (matrix, source server) keeps, for all S destination
//              servers, the prefix sums of the pair's lane-routing tile and traffic tile
//              in LDS (everything the intervals above are made of), then runs through the
//              stages of its source server: with the send offsets known every (stage,
//              source) is independent of the others, so eight lanes - one per lane k of
//              the destination - work out what the stage's chunk of lane k's queue holds
//              for every GPU j, sums over the eight give what each GPU receives, the
//              largest of forwarded and received goes to the stage's scale-up volume
//              with an atomic max.  No lists, no workspace beyond one flag per source;
// rd_matrices  one wavefront per (selected stage, source server) writes the whole
//              G x G matrix.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "k1_rebalance.hpp"

namespace fastk {

constexpr int RD_ROWS = 64;     // source servers per workgroup of rd_offsets (one wavefront)
constexpr int RD_UNROLL = 16;   // stages per batch of the pipelined walk

inline size_t rd_offsets_lds_bytes(int S) { return (size_t)RD_ROWS * S * sizeof(i64); }

__global__ void __launch_bounds__(256) rd_zero(u64* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

// The walk over the stages of a matrix is a chain, but a chain that splits: the stages (in
// execution order) are cut into C chunks, a first kernel adds up what every chunk sends per
// server pair, and the walk of chunk c starts from the sum of the chunks before it.  C is
// chosen by the host so that the chip is full (a batch of 64 matrices of 128 servers has only
// 128 wavefronts otherwise); rd_chunk_len is the number of stages per chunk.
__host__ __device__ inline int rd_chunk_len(int K, int C) {
    const int L = (K + C - 1) / C;
    return (L + RD_UNROLL - 1) / RD_UNROLL * RD_UNROLL;
}

// grid (ceil(S / RD_ROWS), B, C - 1), RD_ROWS threads: what source server a sends to every
// destination in chunk c = blockIdx.z (the last chunk's totals are not needed);
// chunk_tot[b][c][block][d][lane].
template <bool ORDERED>
__global__ void __launch_bounds__(RD_ROWS)
rd_chunk_totals(const int32_t* __restrict__ stages, const i64* __restrict__ stage_bytes,
                const int32_t* __restrict__ num_stages, const int32_t* __restrict__ order,
                i64* __restrict__ chunk_tot, int S, int max_stages) {
    extern __shared__ __align__(16) unsigned char rd_smem[];
    constexpr int U = RD_UNROLL;
    const int b = blockIdx.y, c = blockIdx.z, C = gridDim.z + 1;
    const int lane = threadIdx.x;
    const int a = blockIdx.x * RD_ROWS + lane;
    const int K = min(num_stages[b], max_stages);
    if (K <= 0) return;
    i64* sent = reinterpret_cast<i64*>(rd_smem);                    // [d][lane]
    const int ac = a < S ? a : S - 1;
    for (int d = 0; d < S; ++d) sent[d * RD_ROWS + lane] = 0;
    const int32_t* st = stages + (size_t)b * max_stages * S;
    const i64* by = stage_bytes + (size_t)b * max_stages * S;
    const int32_t* ord = ORDERED ? order + (size_t)b * max_stages : nullptr;
    const int L = rd_chunk_len(K, C);
    const int e0 = min(K, c * L), e1 = min(K, e0 + L);
    // 64 stages per pass: lane u holds the index of the u-th (one coalesced load, a pass ahead),
    // v_readlane hands them out; all 128 row loads of a pass are in flight together, and the
    // fetch-and-adds, whose result nobody reads, queue up in the LDS pipe without a wait
    auto load_idx = [&](int e) -> int {
        const int p = min(e + lane, K - 1);
        if constexpr (ORDERED) return ord[p];
        return p;
    };
    int iv = e0 < e1 ? load_idx(e0) : 0;
    for (int e = e0; e < e1; e += 64) {
        const int cur = iv;
        if (e + 64 < e1) iv = load_idx(e + 64);
        int dd[64];
        i64 ln[64];
#pragma unroll
        for (int u = 0; u < 64; ++u) {
            int s = __builtin_amdgcn_readlane(cur, u);
            s = s < 0 ? 0 : (s >= K ? K - 1 : s);
            dd[u] = e + u < e1 ? st[(size_t)s * S + ac] : -1;
            ln[u] = by[(size_t)s * S + ac];
        }
#pragma unroll
        for (int u = 0; u < 64; ++u) {
            const bool sends = dd[u] >= 0 && dd[u] < S;
            (void)atomicAdd(reinterpret_cast<u64*>(&sent[(sends ? dd[u] : 0) * RD_ROWS + lane]),
                            (u64)(sends ? ln[u] : 0));
        }
    }
    i64* out = chunk_tot + (((size_t)b * (C - 1) + c) * gridDim.x + blockIdx.x) * (size_t)S * RD_ROWS;
    for (int d = 0; d < S; ++d) out[d * RD_ROWS + lane] = sent[d * RD_ROWS + lane];
}

// grid (ceil(S / RD_ROWS), B, C), RD_ROWS threads.  Lane l owns source server a and the
// LDS column [*][l]; no two lanes share a word, so the kernel needs no barrier.
// The walk over the stages of a chunk is a chain of dependent steps (stage index -> the stage's
// row -> the running offset in LDS), so it is software-pipelined by hand: while batch n
// of RD_UNROLL stages is processed, the rows of batch n+1 and the indices of batch n+2
// are in flight.
// ALL: S is a multiple of RD_ROWS, every lane owns a real source server (no store predicate).
template <bool ORDERED, bool ALL>
__global__ void __launch_bounds__(RD_ROWS)
rd_offsets(const int32_t* __restrict__ stages, const i64* __restrict__ stage_bytes,
           const int32_t* __restrict__ num_stages, const int32_t* __restrict__ order,
           const i64* __restrict__ chunk_tot, i64* __restrict__ out_offset, int S, int max_stages) {
    extern __shared__ __align__(16) unsigned char rd_smem[];
    constexpr int U = RD_UNROLL;
    const int b = blockIdx.y, c = blockIdx.z, C = gridDim.z;
    const int lane = threadIdx.x;
    const int a = blockIdx.x * RD_ROWS + lane;
    const int K = min(num_stages[b], max_stages);     // a count beyond the capacity is not trusted
    if (K <= 0) return;
    i64* sent = reinterpret_cast<i64*>(rd_smem);                    // [d][lane]
    const bool live = ALL || a < S;
    const int ac = live ? a : S - 1;                                // clamped: loads stay in range
    // where the chunk starts: what the chunks before it have sent
    // (eight destinations at a time, so that the loads of a pass are in flight together)
    for (int d0 = 0; d0 < S; d0 += 8) {
        i64 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = 0;
        for (int cc = 0; cc < c; ++cc) {
            const i64* tot = chunk_tot + (((size_t)b * (C - 1) + cc) * gridDim.x + blockIdx.x) * (size_t)S * RD_ROWS;
            i64 x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = tot[(size_t)min(d0 + j, S - 1) * RD_ROWS + lane];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] += x[j];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (d0 + j < S) sent[(d0 + j) * RD_ROWS + lane] = v[j];
    }
    const int32_t* st = stages + (size_t)b * max_stages * S;
    const i64* by = stage_bytes + (size_t)b * max_stages * S;
    const int32_t* ord = ORDERED ? order + (size_t)b * max_stages : nullptr;
    i64* off_out = out_offset + (size_t)b * max_stages * S;
    const int L = C > 1 ? rd_chunk_len(K, C) : K;
    const int e_begin = min(K, c * L), e_end = min(K, e_begin + L);

    // one stage: running offset of the pair (a, d) in LDS, send offset out.  Branch-free for
    // an idle row (d < 0): it adds 0 to word 0 of the lane's column.  Lanes beyond S work on a
    // copy of row S-1 in their own LDS column and store nothing.
    auto stage = [&](int s, int d, i64 len) {
        const bool sends = d >= 0 && d < S;
        const int w = (sends ? d : 0) * RD_ROWS + lane;
        const i64 before = (i64)atomicAdd(reinterpret_cast<u64*>(&sent[w]), (u64)(sends ? len : 0));
        if (live) off_out[(size_t)s * S + a] = sends ? before : 0;
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
        bool sends[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            sends[u] = dd[u] >= 0 && dd[u] < S;
            const int w = (sends[u] ? dd[u] : 0) * RD_ROWS + lane;
            off[u] = (i64)atomicAdd(reinterpret_cast<u64*>(&sent[w]), (u64)(sends[u] ? ln[u] : 0));
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (live) off_out[(size_t)ss[u] * S + a] = sends[u] ? off[u] : 0;
    };
    // Three batch buffers take the roles "being processed", "rows in flight", "indices in
    // flight" in turn, so no register is copied while its load is outstanding.
    const int nb = (e_end - e_begin) / U;       // full batches; the tail follows below
    const int eb = e_begin;
    int i0 = 0, i1 = 0, i2 = 0;
    int s0[U], s1[U], s2[U], d0[U], d1[U], d2[U];
    i64 l0[U], l1[U], l2[U];
    if (nb > 0) { i0 = load_idx(eb); load_rows(i0, s0, d0, l0); }
    if (nb > 1) i1 = load_idx(eb + U);
    for (int n = 0; n < nb; n += 3) {
        if (n + 1 < nb) load_rows(i1, s1, d1, l1);
        if (n + 2 < nb) i2 = load_idx(eb + (n + 2) * U);
        process(s0, d0, l0);
        if (n + 1 >= nb) break;
        if (n + 2 < nb) load_rows(i2, s2, d2, l2);
        if (n + 3 < nb) i0 = load_idx(eb + (n + 3) * U);
        process(s1, d1, l1);
        if (n + 2 >= nb) break;
        if (n + 3 < nb) load_rows(i0, s0, d0, l0);
        if (n + 4 < nb) i1 = load_idx(eb + (n + 4) * U);
        process(s2, d2, l2);
    }
    for (int e = eb + nb * U; e < e_end; ++e) {
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
template <int CTRL> __device__ __forceinline__ int rd_dpp_get(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL> __device__ __forceinline__ i64 rd_dpp_get(i64 v) { return dpp_i64<CTRL>(v); }
// largest value among the 8 lanes of a group, in every lane of the group
template <typename I> __device__ __forceinline__ I dpp_max8(I v) {
    v = max(v, rd_dpp_get<0xB1>(v));
    v = max(v, rd_dpp_get<0x4E>(v));
    v = max(v, rd_dpp_get<0x141>(v));
    return v;
}

// Threads per workgroup: the tables of a source server take 512 bytes per destination server
// with 32-bit words, so at 128 servers a compute unit holds them once or twice; sixteen
// wavefronts on one copy keep the unit busier than two workgroups of four on two copies.
constexpr int RV_THREADS32 = 1024;
constexpr int RV_THREADS64 = 256;
constexpr int RV_BLOCK = 128;       // stages a wavefront looks at before it works on those that send
// per destination server: two 8 x 8 tables, and 8 words that keep the pairs of one wavefront's
// 64 consecutive columns on different LDS banks
constexpr int RV_PAIR_WORDS = 136;

// one (stage, source) that sends: destination, stage, offset and length of the chunk
template <typename I> struct alignas(sizeof(I) == 4 ? 16 : 8) rv_entry { int d, s; I off, len; };

template <typename I> inline size_t rd_volumes_lds_bytes(int S) {
    constexpr int waves = (sizeof(I) == 4 ? RV_THREADS32 : RV_THREADS64) / 64;
    return (size_t)S * RV_PAIR_WORDS * sizeof(I) + (size_t)waves * RV_BLOCK * sizeof(rv_entry<I>);
}

// The volumes of all stages in which source server a of matrix b sends.  I: the integer type
// the intervals are worked out in - int when every tile of the source server has a total
// below 2^31 (no offset, prefix sum or overlap can then exceed it), else 64-bit.  Returns false
// (and does nothing) if I is int and the data do not fit.  All threads of the workgroup
// (RV_THREADS32 or RV_THREADS64) call it together.
//
// LDS tables per destination server d, each [i][k] with rows of 8 words (unused rows and
// columns of a cluster with fewer than 8 GPUs per server hold zeros):
//   PX[i][k] = X[i][0] + ... + X[i][k]     (lane-routing tile of the pair, row i)
//   CP[i][j] = t[i][0] + ... + t[i][j]     (traffic tile of the pair, row i)
// Piece (i -> k) has X[i][k] = PX[i][k] - PX[i][k-1] bytes and starts in row i's region at
// PX[i][k-1], plus X[i][i] if the diagonal has not been passed yet (i > k); in lane k's queue
// the pieces follow each other - own head first, then donors in ascending order - so their
// start is a running sum.  The part of a piece that a chunk takes is an interval of the
// region, and what it holds for GPU j is its overlap with [CP[i][j-1], CP[i][j]).
template <typename I>
__device__ __forceinline__ bool
rv_source(const i64* __restrict__ traffic, const i64* __restrict__ X,
          const int32_t* __restrict__ stages, const i64* __restrict__ stage_bytes,
          const i64* __restrict__ stage_offset, u64* __restrict__ redis, int K, int b, int a,
          int S, int G, int max_stages, unsigned char* smem) {
    constexpr int RV_THREADS = sizeof(I) == 4 ? RV_THREADS32 : RV_THREADS64;
    constexpr int RV_WAVES = RV_THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = S * G;
    I* tab = reinterpret_cast<I*>(smem);
    rv_entry<I>* slots = reinterpret_cast<rv_entry<I>*>(tab + (size_t)S * RV_PAIR_WORDS) + wave * RV_BLOCK;

    // ---- the tiles of the source server's G rows (coalesced along the rows), as prefix sums
    bool bad = false;
    if (G == 8) {
        // a tile row is 8 consecutive lanes: its prefix sums by three DPP row shifts, and lane 7
        // of the group collects the row totals of the pair's tile
        const int k8 = tid & 7;
        auto prefix8 = [&](i64 v) -> i64 {
            i64 t = dpp_i64<0x111>(v);      // row_shr:1
            v += k8 >= 1 ? t : 0;
            t = dpp_i64<0x112>(v);          // row_shr:2
            v += k8 >= 2 ? t : 0;
            t = dpp_i64<0x114>(v);          // row_shr:4
            v += k8 >= 4 ? t : 0;
            return v;
        };
        for (int c = tid; c < N; c += RV_THREADS) {
            const int d = c >> 3;
            I* pair = tab + d * RV_PAIR_WORDS + k8;
            i64 x[8], t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const size_t row = ((size_t)b * N + (size_t)a * 8 + i) * N;
                x[i] = X[row + c];
                t[i] = traffic[row + c];
            }
            i64 totx = 0, tott = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if constexpr (sizeof(I) == 4) bad |= (((u64)x[i] | (u64)t[i]) >> 31) != 0;
                const i64 px = prefix8(x[i]), cp = prefix8(t[i]);
                pair[i * 8] = (I)px;
                pair[64 + i * 8] = (I)cp;
                totx += px;
                tott += cp;
            }
            if constexpr (sizeof(I) == 4)
                if (k8 == 7 && d != a) bad |= ((u64)(totx | tott) >> 31) != 0;
        }
    } else {
        for (int e = tid; e < S * RV_PAIR_WORDS; e += RV_THREADS) tab[e] = 0;
        __syncthreads();
        for (int i = 0; i < G; ++i) {
            const size_t row = ((size_t)b * N + (size_t)a * G + i) * N;
            for (int c = tid; c < N; c += RV_THREADS) {
                const int d = c / G;
                const int k = c - d * G;
                const i64 x = X[row + c], t = traffic[row + c];
                if constexpr (sizeof(I) == 4) bad |= (((u64)x | (u64)t) >> 31) != 0;
                tab[d * RV_PAIR_WORDS + i * 8 + k] = (I)x;
                tab[d * RV_PAIR_WORDS + 64 + i * 8 + k] = (I)t;
            }
        }
        __syncthreads();
        // prefix sums along every row, in place: thread (d, i); the 8 threads of a pair add up
        // its total
        for (int it = tid; it < S * 8; it += RV_THREADS) {
            const int d = it >> 3, i = it & 7;
            I* px = tab + d * RV_PAIR_WORDS + i * 8;
            I* cp = px + 64;
            i64 sx = 0, st = 0;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                sx += (i64)px[k];
                px[k] = (I)sx;
                st += (i64)cp[k];
                cp[k] = (I)st;
            }
            if constexpr (sizeof(I) == 4) {
                sx = dpp_sum8(sx);
                st = dpp_sum8(st);
                if (d != a) bad |= ((u64)(sx | st) >> 31) != 0;
            }
        }
    }
    if (__syncthreads_or(bad ? 1 : 0)) {
        if constexpr (sizeof(I) == 4) return false;
    }

    // ---- the stages.  A wavefront takes RV_BLOCK stages at a time, files the ones in which
    // the source server sends (on skewed traffic most rows of a stage carry virtual bytes only)
    // in its LDS slots, and works on eight of them at once: lane (g, k) = lane k of entry g.
    const int grp = lane >> 3, k = lane & 7;
    const int km = k > 0 ? k - 1 : 0;
    const size_t base = (size_t)b * max_stages * S + a;
    const int32_t* st = stages + base;
    const i64* by = stage_bytes + base;
    const i64* of = stage_offset + base;
    // the destinations of a block are loaded one block ahead of their use (a strided walk down
    // the column of the source server: every load is a round trip to L2 or further); offsets
    // and lengths only where the source server sends - loading them for every stage costs more
    // memory traffic than the wait it hides
    constexpr int H = RV_BLOCK / 64;
    int dn[H];
    auto fetch = [&](int s0) {
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const int s = s0 + h * 64 + lane;
            dn[h] = -1;
            if (s < K) dn[h] = st[(size_t)s * S];
        }
    };
    if (wave * RV_BLOCK < K) fetch(wave * RV_BLOCK);
    for (int s0 = wave * RV_BLOCK; s0 < K; s0 += RV_WAVES * RV_BLOCK) {
        int dc[H];
#pragma unroll
        for (int h = 0; h < H; ++h) dc[h] = dn[h];
        if (s0 + RV_WAVES * RV_BLOCK < K) fetch(s0 + RV_WAVES * RV_BLOCK);
        int n = 0;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const int d = dc[h];
            const int s = s0 + h * 64 + lane;
            const bool act = d >= 0 && d < S && d != a;
            const u64 m = __builtin_amdgcn_ballot_w64(act);
            if (act) {
                const int r = n + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                      __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                rv_entry<I> e;
                e.d = d;
                e.s = s;
                e.off = (I)of[(size_t)s * S];
                e.len = (I)by[(size_t)s * S];
                slots[r] = e;
            }
            n += __builtin_popcountll(m);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // the wavefront's own slots
        __builtin_amdgcn_wave_barrier();
        for (int e0 = 0; e0 < n; e0 += 8) {
            const bool valid = e0 + grp < n;
            const rv_entry<I> e = slots[valid ? e0 + grp : n - 1];
            const I off = e.off;
            const I end = off + (valid && e.len > 0 ? e.len : (I)0);
            const I* T = tab + e.d * RV_PAIR_WORDS;
            I recv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) recv[j] = 0;
            // the part [ua, ub) of row i's region: what it holds for every GPU j
            auto spread = [&](const I* cp, I ua, I ub) {
                I c[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) c[j] = cp[j];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const I lo = j > 0 ? max(ua, c[j - 1]) : ua;
                    const I hi = min(ub, c[j]);
                    recv[j] += max(hi - lo, (I)0);
                }
            };
            // own head first: piece (k -> k), at the start of the queue and of the region
            I q;
            {
                const I* px = T + k * 8;
                const I pk = px[k], pm = px[km];
                q = pk - (k > 0 ? pm : (I)0);
                const I hi = min(end, q);
                spread(px + 64, min(off, hi), hi);
            }
            // then the pieces handed in, in ascending donor index
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const I* px = T + i * 8;
                const I pk = px[k], pm0 = px[km];
                const I pm = k > 0 ? pm0 : (I)0;
                const I len = i == k ? (I)0 : pk - pm;
                const I lo = max(off, q), hi = min(end, q + len);
                const bool hit = hi > lo;
                if (__builtin_amdgcn_ballot_w64(hit) != 0) {
                    // a lane whose chunk misses the piece passes the empty interval [0, 0): its
                    // own offsets are out of the piece's range and must not enter the arithmetic
                    const I xii = px[i] - (i > 0 ? px[i - 1] : (I)0);
                    const I ua = hit ? pm + (i > k ? xii : (I)0) + (lo - q) : (I)0;
                    spread(px + 64, ua, hit ? ua + (hi - lo) : (I)0);
                }
                q += len;
            }
            // what the lane forwards (everything that is not for its own GPU), what every GPU
            // is sent by the other lanes, and the largest of all
            I fwd = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                recv[j] = j == k ? (I)0 : recv[j];
                fwd += recv[j];
            }
            I v = dpp_max8<I>(fwd);
#pragma unroll
            for (int j = 0; j < 8; ++j) v = max(v, dpp_sum8(recv[j]));
            if (k == 0 && valid && v > 0) atomicMax(&redis[e.s], (u64)v);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // slots read before they are refilled
        __builtin_amdgcn_wave_barrier();
    }
    return true;
}

// Maps a workgroup index to a (matrix, source server) item so that the 16 consecutive source
// servers whose stage rows share cache lines run on the same XCD at about the same time
// (workgroups are dealt to the 8 XCDs in turn, and each XCD has its own L2).
__device__ __forceinline__ int rv_item(int idx) {
    const int xcd = idx & 7, slot = idx >> 3;
    return ((slot >> 4) * 8 + xcd) * 16 + (slot & 15);
}
inline unsigned rv_grid(int items) { return (unsigned)((items + 127) / 128 * 128); }

// grid rv_grid(B * S), RV_THREADS32 threads, LDS rd_volumes_lds_bytes<int>(S): 32-bit intervals;
// need64[b * S + a] = 1 where the source server's data do not fit (0 otherwise).
__global__ void __launch_bounds__(RV_THREADS32)
rd_volumes32(const i64* __restrict__ traffic, const i64* __restrict__ X,
             const int32_t* __restrict__ stages, const i64* __restrict__ stage_bytes,
             const i64* __restrict__ stage_offset, const int32_t* __restrict__ num_stages,
             int32_t* __restrict__ need64, u64* __restrict__ redis, int B, int S, int G,
             int max_stages) {
    extern __shared__ __align__(16) unsigned char rv_smem[];
    const int item = rv_item((int)blockIdx.x);
    if (item >= B * S) return;
    const int b = item / S, a = item - b * S;
    const int K = min(num_stages[b], max_stages);
    if (K <= 0) return;
    const bool ok = rv_source<int>(traffic, X, stages, stage_bytes, stage_offset,
                                   redis + (size_t)b * max_stages, K, b, a, S, G, max_stages, rv_smem);
    if (threadIdx.x == 0) need64[item] = ok ? 0 : 1;
}

// grid <= B * S, RV_THREADS64 threads, LDS rd_volumes_lds_bytes<i64>(S): the source servers that
// rd_volumes32 left, with 64-bit intervals.  Each workgroup goes through its share of the items.
__global__ void __launch_bounds__(RV_THREADS64)
rd_volumes64(const i64* __restrict__ traffic, const i64* __restrict__ X,
             const int32_t* __restrict__ stages, const i64* __restrict__ stage_bytes,
             const i64* __restrict__ stage_offset, const int32_t* __restrict__ num_stages,
             const int32_t* __restrict__ need64, u64* __restrict__ redis, int B, int S, int G,
             int max_stages) {
    extern __shared__ __align__(16) unsigned char rv_smem[];
    for (int item = (int)blockIdx.x; item < B * S; item += (int)gridDim.x) {
        const int b = item / S, a = item - b * S;
        const int K = min(num_stages[b], max_stages);
        if (K <= 0 || need64[item] == 0) continue;      // the same for every thread
        (void)rv_source<i64>(traffic, X, stages, stage_bytes, stage_offset,
                             redis + (size_t)b * max_stages, K, b, a, S, G, max_stages, rv_smem);
        __syncthreads();        // the tables are rebuilt for the next item
    }
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
