// Host side of the C ABI declared in include/fast.h: argument checks, the plan's
// device workspaces, and the kernel launches of every entry point.
#include "fast.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>
#include <new>

#include "k1_rebalance.hpp"
#include "decompose.hpp"
#include "k3_cost.hpp"
#include "k4_spreadout.hpp"
#include "k5_build_traffic.hpp"
#include "k6_stage_order.hpp"
#include "k7_redistribution.hpp"
#include "k8_pipeline.hpp"

using fastk::i64;

// Workspace of fast_synthesize_batched_noalloc: every GPU the library runs on holds its own
// copy of this array, at its own address, until the process ends.  Host code never uses the
// array's name as an address: scratch_address() asks the runtime for the device address once
// per device and everything else goes through that pointer.
static __device__ __align__(256) unsigned char scratch[FAST_NOALLOC_SCRATCH_BYTES];

struct fast_plan {
    int S, G;
    double bw_up, bw_out;
    double delay;  // link wake-up delay per executed step, seconds
    int matching;  // FAST_MATCHING_*: which decomposition kernel the synthesis call runs
    int device;
    int max_stages;
    // device workspace for `cap_B` matrices
    int cap_B;
    i64* wsT;      // [B][S][S]  server-to-server totals
    i64* wsQ;      // [B][S][S]  per-lane server-level matrix
    i64* wsPart;   // [B][S][K1_PART]
    i64* wsC;      // [B][max_stages] stage weights
    // workspace of the SpreadOut baseline for `spo_cap_B` matrices
    int spo_cap_B;
    fastk::u64* spoDiag;   // [B][2][N] per-diagonal maxima
    i64* spoT;             // [B][S][S]
    int* spoNeg;           // [B][chunks]
    // workspace of the stage-order sort for `so_cap_B` matrices
    int so_cap_B;
    fastk::u64* soKeys;    // [B][P]
    int32_t* soIdx;        // [B][P]
    // workspace of the redistribution analysis for `rd_cap_B` matrices
    int rd_cap_B;
    int32_t* rdNeed;       // [B][S] 1 where a source server's tiles need 64-bit intervals
    // workspace of the chunked stage walk
    size_t rd_chunk_bytes;
    i64* rdChunk;          // [B][C - 1][blocks][S][64] bytes sent per server pair in each chunk
    int last_B;            // B of the most recent synthesis call (0 = none)
    unsigned char* scratch_ptr;   // device address of `scratch` on the plan's device
    // timing: four events per recorded call
    int timing;
    int n_timed;
    hipEvent_t (*ev)[4];
};

namespace {

// The four workspace arrays of a synthesis call for B matrices, wherever they live.
struct synth_workspace {
    i64* T;      // [B][S][S]  server-to-server totals
    i64* Q;      // [B][S][S]  per-lane server-level matrix
    i64* Part;   // [B][S][K1_PART]
    i64* C;      // [B][max_stages] stage weights
};

void free_workspace(fast_plan* p) {
    if (p->wsT) (void)hipFree(p->wsT);
    p->wsT = p->wsQ = p->wsPart = p->wsC = nullptr;
    p->cap_B = 0;
}

void free_spo_workspace(fast_plan* p) {
    if (p->spoDiag) (void)hipFree(p->spoDiag);
    p->spoDiag = nullptr;
    p->spoT = nullptr;
    p->spoNeg = nullptr;
    p->spo_cap_B = 0;
}

int grow_spo_workspace(fast_plan* p, int B) {
    if (B <= p->spo_cap_B) return FAST_OK;
    free_spo_workspace(p);
    const size_t S = p->S, N = (size_t)p->S * p->G;
    const size_t chunks = (S + fastk::spo_chunk_servers(p->S, p->G) - 1) /
                          fastk::spo_chunk_servers(p->S, p->G);
    const size_t nDiag = (size_t)B * 2 * N, nT = (size_t)B * S * S, nNeg = (size_t)B * chunks;
    unsigned char* base = nullptr;
    if (hipMalloc(&base, (nDiag + nT) * sizeof(i64) + nNeg * sizeof(int)) != hipSuccess) {
        (void)hipGetLastError();
        return FAST_ERR_OOM;
    }
    p->spoDiag = reinterpret_cast<fastk::u64*>(base);
    p->spoT = reinterpret_cast<i64*>(p->spoDiag + nDiag);
    p->spoNeg = reinterpret_cast<int*>(p->spoT + nT);
    p->spo_cap_B = B;
    return FAST_OK;
}

template <int G>
void launch_spo_scan(const fast_plan* p, int B, const i64* traffic, int CS, int chunks,
                     hipStream_t stream) {
    const dim3 grid(chunks, B), block(fastk::SPO_THREADS);
    const size_t lds = fastk::spo_scan_lds_bytes(p->S, G);
    if constexpr (G % 2 == 0) {
        if (reinterpret_cast<uintptr_t>(traffic) % 16 == 0) {
            hipLaunchKernelGGL((fastk::spo_scan<G, true>), grid, block, lds, stream, traffic,
                               p->spoDiag, p->spoT, p->spoNeg, p->S, CS);
            return;
        }
    }
    hipLaunchKernelGGL((fastk::spo_scan<G, false>), grid, block, lds, stream, traffic, p->spoDiag,
                       p->spoT, p->spoNeg, p->S, CS);
}

int grow_workspace(fast_plan* p, int B) {
    if (B <= p->cap_B) return FAST_OK;
    free_workspace(p);
    const size_t S = p->S;
    const size_t nT = (size_t)B * S * S, nPart = (size_t)B * S * fastk::K1_PART,
                 nC = (size_t)B * p->max_stages;
    i64* base = nullptr;
    if (hipMalloc(&base, (2 * nT + nPart + nC) * sizeof(i64)) != hipSuccess) {
        (void)hipGetLastError();
        return FAST_ERR_OOM;
    }
    p->wsT = base;
    p->wsQ = base + nT;
    p->wsPart = p->wsQ + nT;
    p->wsC = p->wsPart + nPart;
    p->cap_B = B;
    return FAST_OK;
}

static_assert(fastk::K1_MAX_S == FAST_MAX_SERVERS, "kernel 1 unrolls for FAST_MAX_SERVERS");

template <int G>
void launch_k1(const fast_plan* p, const synth_workspace& ws, int B, const i64* traffic, i64* X,
               hipStream_t stream) {
    const dim3 grid(p->S, B), block(fastk::K1_THREADS);
    const size_t lds = fastk::k1_lds_bytes(p->S, G);
    const bool vec = (G % 2 == 0) && ((reinterpret_cast<uintptr_t>(traffic) |
                                       reinterpret_cast<uintptr_t>(X)) % 16 == 0);
    if constexpr (G == 2 || G == 4 || G == 8) {
        if (vec) {
            hipLaunchKernelGGL((fastk::k1_rebalance_tiles<G>), grid, block,
                               fastk::k1_tiles_lds_bytes(G), stream, traffic, X, ws.T, ws.Q,
                               ws.Part, p->S);
            return;
        }
    } else if constexpr (G % 2 == 0) {
        if (vec) {
            hipLaunchKernelGGL((fastk::k1_rebalance<G, true>), grid, block, lds, stream, traffic,
                               X, ws.T, ws.Q, ws.Part, p->S);
            return;
        }
    }
    hipLaunchKernelGGL((fastk::k1_rebalance<G, false>), grid, block, lds, stream, traffic, X,
                       ws.T, ws.Q, ws.Part, p->S);
}


// The stage-walk kernel: with or without a stage order, and the variant without store predicates
// when S is a multiple of its 64 source servers per wavefront.
typedef void (*rd_offsets_fn)(const int32_t*, const i64*, const int32_t*, const int32_t*, const i64*,
                              i64*, int, int);
rd_offsets_fn rd_offsets_kernel(int S, bool ordered) {
    const bool all = S % fastk::RD_ROWS == 0;
    if (ordered) return all ? &fastk::rd_offsets<true, true> : &fastk::rd_offsets<true, false>;
    return all ? &fastk::rd_offsets<false, true> : &fastk::rd_offsets<false, false>;
}

// Chunks the stage walk of B matrices is cut into: enough wavefronts to occupy the chip (a
// wavefront covers 64 source servers and keeps 512 * S bytes of LDS), at least 256 stages of
// capacity per chunk, at most 16.
int rd_chunks(const fast_plan* p, int B) {
    const long waves = (long)B * ((p->S + fastk::RD_ROWS - 1) / fastk::RD_ROWS);
    long c = (512 + waves - 1) / waves;
    const long by_len = p->max_stages / 256;
    if (c > by_len) c = by_len;
    if (c > 16) c = 16;
    return c < 1 ? 1 : (int)c;
}

// The per-pair totals of the chunks: `units` tables of S x 64 words (one per matrix, chunk but
// the last, and block of 64 source servers).
int grow_chunk_workspace(fast_plan* p, size_t units) {
    const size_t need = units * p->S * fastk::RD_ROWS * sizeof(i64);
    if (need <= p->rd_chunk_bytes) return FAST_OK;
    if (p->rdChunk) (void)hipFree(p->rdChunk);
    p->rdChunk = nullptr;
    p->rd_chunk_bytes = 0;
    if (hipMalloc(&p->rdChunk, need) != hipSuccess) {
        (void)hipGetLastError();
        p->rdChunk = nullptr;
        return FAST_ERR_OOM;
    }
    p->rd_chunk_bytes = need;
    return FAST_OK;
}

// One flag per source server of B matrices (which of them need 64-bit intervals).
int grow_rd_workspace(fast_plan* p, int B) {
    if (B <= p->rd_cap_B) return FAST_OK;
    if (p->rdNeed) (void)hipFree(p->rdNeed);
    p->rdNeed = nullptr;
    p->rd_cap_B = 0;
    if (hipMalloc(&p->rdNeed, (size_t)B * p->S * sizeof(int32_t)) != hipSuccess) {
        (void)hipGetLastError();
        p->rdNeed = nullptr;
        return FAST_ERR_OOM;
    }
    p->rd_cap_B = B;
    return FAST_OK;
}

int next_pow2(int v);

// Keys and indices of the stage-order sort for B matrices.
int grow_so_workspace(fast_plan* p, int B) {
    if (B <= p->so_cap_B) return FAST_OK;
    const int P = next_pow2(p->max_stages);
    if (p->soKeys) (void)hipFree(p->soKeys);
    p->soKeys = nullptr;
    p->so_cap_B = 0;
    unsigned char* base = nullptr;
    if (hipMalloc(&base, (size_t)B * P * (sizeof(i64) + sizeof(int32_t))) != hipSuccess) {
        (void)hipGetLastError();
        return FAST_ERR_OOM;
    }
    p->soKeys = reinterpret_cast<fastk::u64*>(base);
    p->soIdx = reinterpret_cast<int32_t*>(p->soKeys + (size_t)B * P);
    p->so_cap_B = B;
    return FAST_OK;
}

// Enqueues the send offsets of B matrices (chunk totals first when the walk is cut up).
int launch_stage_offsets(fast_plan* p, int B, const int32_t* stages, const int64_t* stage_bytes,
                         const int32_t* num_stages, const int32_t* stage_order,
                         int64_t* out_stage_offset, hipStream_t stream) {
    const int C = rd_chunks(p, B);
    const unsigned blocks = (unsigned)((p->S + fastk::RD_ROWS - 1) / fastk::RD_ROWS);
    const size_t lds = fastk::rd_offsets_lds_bytes(p->S);
    if (C > 1) {
        if (const int rc = grow_chunk_workspace(p, (size_t)B * (C - 1) * blocks); rc != FAST_OK)
            return rc;
        const dim3 grid1(blocks, B, C - 1);
        if (stage_order)
            hipLaunchKernelGGL(fastk::rd_chunk_totals<true>, grid1, dim3(fastk::RD_ROWS), lds, stream,
                               stages, reinterpret_cast<const i64*>(stage_bytes), num_stages,
                               stage_order, p->rdChunk, p->S, p->max_stages);
        else
            hipLaunchKernelGGL(fastk::rd_chunk_totals<false>, grid1, dim3(fastk::RD_ROWS), lds, stream,
                               stages, reinterpret_cast<const i64*>(stage_bytes), num_stages,
                               stage_order, p->rdChunk, p->S, p->max_stages);
    }
    hipLaunchKernelGGL(rd_offsets_kernel(p->S, stage_order != nullptr), dim3(blocks, B, C),
                       dim3(fastk::RD_ROWS), lds, stream, stages,
                       reinterpret_cast<const i64*>(stage_bytes), num_stages, stage_order,
                       C > 1 ? p->rdChunk : nullptr, reinterpret_cast<i64*>(out_stage_offset), p->S,
                       p->max_stages);
    return FAST_OK;
}

// Device address of `scratch` on device `dev`, which has to be the current device; looked up
// once per device.
constexpr int SCRATCH_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[SCRATCH_MAX_DEVICES];

int scratch_address(int dev, unsigned char** out) {
    if (dev < 0 || dev >= SCRATCH_MAX_DEVICES) return FAST_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        unsigned char* ptr = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess ||
            !ptr) {
            (void)hipGetLastError();
            return FAST_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return FAST_OK;
}

// FAST_OK if the plan's device is the current one (the kernels would otherwise be launched
// on another GPU than the one that holds the workspace), else the error to return.
int check_device(const fast_plan* p) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return FAST_ERR_HIP;
    }
    return dev == p->device ? FAST_OK : FAST_ERR_INVALID_ARG;
}

int next_pow2(int v) {
    int n = 1;
    while (n < v) n <<= 1;
    return n;
}

// Enqueues the kernels of one synthesis call (aggregation + balancing, decomposition, cost
// model) on `stream`; ev = four events to record around them, or nullptr.
void enqueue_synthesis(const fast_plan* p, const synth_workspace& ws, int B, const int64_t* traffic,
                       int64_t* out_rebalance, int32_t* out_stages, int64_t* out_stage_bytes,
                       int32_t* out_num_stages, double* out_predicted_time, hipEvent_t* ev,
                       hipStream_t stream) {
    if (ev) (void)hipEventRecord(ev[0], stream);
    const i64* tr = reinterpret_cast<const i64*>(traffic);
    i64* X = reinterpret_cast<i64*>(out_rebalance);
    switch (p->G) {
        case 1: launch_k1<1>(p, ws, B, tr, X, stream); break;
        case 2: launch_k1<2>(p, ws, B, tr, X, stream); break;
        case 3: launch_k1<3>(p, ws, B, tr, X, stream); break;
        case 4: launch_k1<4>(p, ws, B, tr, X, stream); break;
        case 5: launch_k1<5>(p, ws, B, tr, X, stream); break;
        case 6: launch_k1<6>(p, ws, B, tr, X, stream); break;
        case 7: launch_k1<7>(p, ws, B, tr, X, stream); break;
        default: launch_k1<8>(p, ws, B, tr, X, stream); break;
    }
    if (ev) (void)hipEventRecord(ev[1], stream);

    i64* sb = reinterpret_cast<i64*>(out_stage_bytes);
    const bool slow_up = p->bw_up < (double)(p->G - 1) * p->bw_out;
    const int sort_n = slow_up ? next_pow2(p->max_stages) : 0;
    // Small clusters are bound by the launches: there the cost model rides on the decomposition
    // kernel's wavefront (about 3 us less per call), unless it has to sort the stage weights
    // (slow scale-up fabric) or the fewer-stages kernel is in use.  On large clusters one
    // wavefront takes longer over the model's reductions than kernel 3's launch costs.
    const bool with_cost =
        p->matching == FAST_MATCHING_SUPPORT && sort_n == 0 && p->S <= fastk::K2_COST_MAX_S;
    if (p->matching == FAST_MATCHING_BOTTLENECK)
        fastk::launch_k9(p->S, B, stream, ws.Q, ws.Part, out_stages, sb, out_num_stages, ws.C,
                         p->max_stages);
    else
        fastk::launch_k2(p->S, with_cost, B, stream, ws.Q, ws.Part, out_stages, sb,
                         out_num_stages, ws.C, p->max_stages, ws.T, out_predicted_time, p->G,
                         p->bw_up, p->bw_out, p->delay);
    if (ev) (void)hipEventRecord(ev[2], stream);

    if (!with_cost)
        hipLaunchKernelGGL(fastk::k3_cost, dim3(B), dim3(fastk::K3_THREADS),
                           (size_t)sort_n * sizeof(i64), stream, ws.T, ws.Part, ws.C,
                           out_num_stages, out_predicted_time, p->S, p->G, p->max_stages, p->bw_up,
                           p->bw_out, p->delay, sort_n);
    if (ev) (void)hipEventRecord(ev[3], stream);
}

}  // namespace

extern "C" {

int fast_plan_create(int S, int G, double link_bw_up, double link_bw_out, fast_plan_t** out_plan) {
    if (!out_plan) return FAST_ERR_INVALID_ARG;
    *out_plan = nullptr;
    if (S < 1 || G < 1) return FAST_ERR_INVALID_ARG;
    if (!std::isfinite(link_bw_up) || !std::isfinite(link_bw_out) || link_bw_up <= 0.0 ||
        link_bw_out <= 0.0)
        return FAST_ERR_INVALID_ARG;
    if (S > FAST_MAX_SERVERS || G > FAST_MAX_GPUS_PER_SERVER) return FAST_ERR_UNSUPPORTED;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return FAST_ERR_HIP;
    }
    fast_plan* p = new (std::nothrow) fast_plan();
    if (!p) return FAST_ERR_OOM;
    p->S = S;
    p->G = G;
    p->bw_up = link_bw_up;
    p->bw_out = link_bw_out;
    p->device = dev;
    p->max_stages = S * S;
    p->delay = 0.0;
    p->matching = FAST_MATCHING_SUPPORT;
    p->cap_B = 0;
    p->wsT = p->wsQ = p->wsPart = p->wsC = nullptr;
    p->spo_cap_B = 0;
    p->spoDiag = nullptr;
    p->spoT = nullptr;
    p->spoNeg = nullptr;
    p->so_cap_B = 0;
    p->soKeys = nullptr;
    p->soIdx = nullptr;
    p->rd_cap_B = 0;
    p->rdNeed = nullptr;
    p->rd_chunk_bytes = 0;
    p->rdChunk = nullptr;
    p->last_B = 0;
    p->scratch_ptr = nullptr;
    p->timing = 0;
    p->n_timed = 0;
    p->ev = nullptr;

    if (const int rc = scratch_address(dev, &p->scratch_ptr); rc != FAST_OK) {
        delete p;
        return rc;
    }
    hipError_t e = fastk::decompose_prepare(S);
    if (e == hipSuccess && link_bw_up < (double)(G - 1) * link_bw_out)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fastk::k3_cost),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)(next_pow2(p->max_stages) * sizeof(i64)));
    if (e == hipSuccess && fastk::rd_offsets_lds_bytes(S) > 48 * 1024) {
        for (int k = 0; k < 2 && e == hipSuccess; ++k)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(rd_offsets_kernel(S, k == 0)),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)fastk::rd_offsets_lds_bytes(S));
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fastk::rd_chunk_totals<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)fastk::rd_offsets_lds_bytes(S));
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fastk::rd_chunk_totals<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)fastk::rd_offsets_lds_bytes(S));
    }
    if (e == hipSuccess && fastk::rd_volumes_lds_bytes<int>(S) > 48 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fastk::rd_volumes32),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)fastk::rd_volumes_lds_bytes<int>(S));
    if (e == hipSuccess && fastk::rd_volumes_lds_bytes<i64>(S) > 48 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fastk::rd_volumes64),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)fastk::rd_volumes_lds_bytes<i64>(S));
    if (e != hipSuccess) {
        (void)hipGetLastError();
        delete p;
        return FAST_ERR_HIP;
    }
    *out_plan = p;
    return FAST_OK;
}

int fast_plan_max_stages(const fast_plan_t* plan) { return plan ? plan->max_stages : -1; }

int fast_synthesize_batched(fast_plan_t* p, int B, const int64_t* traffic, int64_t* out_rebalance,
                            int32_t* out_stages, int64_t* out_stage_bytes, int32_t* out_num_stages,
                            double* out_predicted_time, hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!traffic || !out_rebalance || !out_stages || !out_stage_bytes || !out_num_stages ||
        !out_predicted_time)
        return FAST_ERR_INVALID_ARG;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;     // grid.y limit of the first kernel
    int rc = check_device(p);
    if (rc != FAST_OK) return rc;
    rc = grow_workspace(p, B);
    if (rc != FAST_OK) return rc;

    hipEvent_t* ev = nullptr;
    if (p->timing && p->n_timed < FAST_MAX_TIMED_CALLS) {
        if (!p->ev) {
            p->ev = new (std::nothrow) hipEvent_t[FAST_MAX_TIMED_CALLS][4]();
            if (!p->ev) return FAST_ERR_OOM;
        }
        ev = p->ev[p->n_timed];
        for (int k = 0; k < 4; ++k)
            if (!ev[k] && hipEventCreate(&ev[k]) != hipSuccess) {
                (void)hipGetLastError();
                return FAST_ERR_HIP;
            }
    }
    const synth_workspace ws = {p->wsT, p->wsQ, p->wsPart, p->wsC};
    enqueue_synthesis(p, ws, B, traffic, out_rebalance, out_stages, out_stage_bytes, out_num_stages,
                      out_predicted_time, ev, stream);
    if (ev) ++p->n_timed;
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    p->last_B = B;
    return FAST_OK;
}

int fast_synthesize_batched_noalloc(fast_plan_t* p, int B, const int64_t* traffic,
                                    int64_t* out_rebalance, int32_t* out_stages,
                                    int64_t* out_stage_bytes, int32_t* out_num_stages,
                                    double* out_predicted_time, hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!traffic || !out_rebalance || !out_stages || !out_stage_bytes || !out_num_stages ||
        !out_predicted_time)
        return FAST_ERR_INVALID_ARG;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    // the same four arrays as the plan's workspace, carved out of the static array; every one
    // of them is written in full by the kernels before it is read, so nothing has to be cleared
    const size_t S = p->S;
    const size_t nT = (size_t)B * S * S, nPart = (size_t)B * S * fastk::K1_PART,
                 nC = (size_t)B * p->max_stages;
    if ((2 * nT + nPart + nC) * sizeof(i64) > (size_t)FAST_NOALLOC_SCRATCH_BYTES)
        return FAST_ERR_UNSUPPORTED;
    i64* base = reinterpret_cast<i64*>(p->scratch_ptr);
    const synth_workspace ws = {base, base + nT, base + 2 * nT, base + 2 * nT + nPart};
    enqueue_synthesis(p, ws, B, traffic, out_rebalance, out_stages, out_stage_bytes, out_num_stages,
                      out_predicted_time, nullptr, stream);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_plan_set_wakeup_delay(fast_plan_t* p, double seconds) {
    if (!p || !std::isfinite(seconds) || seconds < 0.0) return FAST_ERR_INVALID_ARG;
    p->delay = seconds;
    return FAST_OK;
}

int fast_plan_set_matching(fast_plan_t* p, int matching) {
    if (!p || (matching != FAST_MATCHING_SUPPORT && matching != FAST_MATCHING_BOTTLENECK))
        return FAST_ERR_INVALID_ARG;
    p->matching = matching;
    return FAST_OK;
}

int fast_spreadout_batched(fast_plan_t* p, int B, const int64_t* traffic,
                           double* out_spreadout_time, hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!traffic || !out_spreadout_time) return FAST_ERR_INVALID_ARG;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    int rc = check_device(p);
    if (rc != FAST_OK) return rc;
    rc = grow_spo_workspace(p, B);
    if (rc != FAST_OK) return rc;
    const int N = p->S * p->G;
    const int CS = fastk::spo_chunk_servers(p->S, p->G);
    const int chunks = (p->S + CS - 1) / CS;
    const size_t nDiag = (size_t)B * 2 * N;
    // the per-diagonal maxima are merged with atomic max, so they start from zero
    // (a fill kernel, not a memset node, so that the call can be captured in a graph)
    hipLaunchKernelGGL(fastk::spo_zero, dim3((unsigned)((nDiag + 1023) / 1024 < 1024
                                                           ? (nDiag + 1023) / 1024 : 1024)),
                       dim3(256), 0, stream, p->spoDiag, nDiag);
    const i64* tr = reinterpret_cast<const i64*>(traffic);
    switch (p->G) {
        case 1: launch_spo_scan<1>(p, B, tr, CS, chunks, stream); break;
        case 2: launch_spo_scan<2>(p, B, tr, CS, chunks, stream); break;
        case 3: launch_spo_scan<3>(p, B, tr, CS, chunks, stream); break;
        case 4: launch_spo_scan<4>(p, B, tr, CS, chunks, stream); break;
        case 5: launch_spo_scan<5>(p, B, tr, CS, chunks, stream); break;
        case 6: launch_spo_scan<6>(p, B, tr, CS, chunks, stream); break;
        case 7: launch_spo_scan<7>(p, B, tr, CS, chunks, stream); break;
        default: launch_spo_scan<8>(p, B, tr, CS, chunks, stream); break;
    }
    hipLaunchKernelGGL(fastk::spo_finish, dim3(B), dim3(fastk::SPO_THREADS),
                       (size_t)N * sizeof(double), stream, p->spoDiag, p->spoT, p->spoNeg,
                       out_spreadout_time, p->S, p->G, chunks, p->bw_up, p->bw_out, p->delay);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_stage_order_batched(fast_plan_t* p, int B, const int64_t* stage_bytes,
                             const int32_t* num_stages, int32_t* out_stage_order,
                             hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!stage_bytes || !num_stages || !out_stage_order) return FAST_ERR_INVALID_ARG;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    const int P = next_pow2(p->max_stages);
    if (const int rc = grow_so_workspace(p, B); rc != FAST_OK) return rc;
    const int per = fastk::SO_W_THREADS / 64;
    hipLaunchKernelGGL(fastk::so_weights, dim3((P + per - 1) / per, B), dim3(fastk::SO_W_THREADS),
                       0, stream, reinterpret_cast<const i64*>(stage_bytes), num_stages,
                       p->soKeys, p->soIdx, p->S, p->max_stages, P);
    hipLaunchKernelGGL(fastk::so_sort, dim3(B), dim3(fastk::SO_THREADS), 0, stream, p->soKeys,
                       p->soIdx, num_stages, out_stage_order, p->max_stages, P);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_build_traffic_batched(fast_plan_t* p, int B, int E, const int64_t* tokens_per_expert,
                               const int32_t* expert_to_gpu, int64_t token_bytes,
                               int64_t* out_traffic, int32_t* out_status, hipStream_t stream) {
    if (!p || B < 0 || E < 1 || token_bytes <= 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!tokens_per_expert || !expert_to_gpu || !out_traffic || !out_status)
        return FAST_ERR_INVALID_ARG;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    const int N = p->S * p->G;
    hipLaunchKernelGGL(fastk::bt_zero, dim3((B + 255) / 256), dim3(256), 0, stream, out_status, B);
    hipLaunchKernelGGL(fastk::bt_build, dim3(N, B), dim3(fastk::BT_THREADS),
                       (size_t)N * sizeof(i64), stream,
                       reinterpret_cast<const i64*>(tokens_per_expert), expert_to_gpu,
                       reinterpret_cast<i64*>(out_traffic), out_status, N, E, (i64)token_bytes);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_stage_offsets_batched(fast_plan_t* p, int B, const int32_t* stages,
                               const int64_t* stage_bytes, const int32_t* num_stages,
                               const int32_t* stage_order, int64_t* out_stage_offset,
                               hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!stages || !stage_bytes || !num_stages || !out_stage_offset) return FAST_ERR_INVALID_ARG;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    if (const int rc = launch_stage_offsets(p, B, stages, stage_bytes, num_stages, stage_order,
                                            out_stage_offset, stream);
        rc != FAST_OK)
        return rc;
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_redistribution_batched(fast_plan_t* p, int B, const int64_t* traffic,
                                const int64_t* rebalance, const int32_t* stages,
                                const int64_t* stage_bytes, const int32_t* num_stages,
                                const int32_t* stage_order, int64_t* out_stage_offset,
                                int64_t* out_redis_bytes, hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!traffic || !rebalance || !stages || !stage_bytes || !num_stages || !out_stage_offset ||
        !out_redis_bytes)
        return FAST_ERR_INVALID_ARG;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    const size_t M = p->max_stages;
    if (const int rc = grow_rd_workspace(p, B); rc != FAST_OK) return rc;
    const size_t nR = (size_t)B * M;
    fastk::u64* redis = reinterpret_cast<fastk::u64*>(out_redis_bytes);
    hipLaunchKernelGGL(fastk::rd_zero, dim3((unsigned)((nR + 255) / 256 < 2048 ? (nR + 255) / 256
                                                                              : 2048)),
                       dim3(256), 0, stream, redis, nR);
    if (const int rc = launch_stage_offsets(p, B, stages, stage_bytes, num_stages, stage_order,
                                            out_stage_offset, stream);
        rc != FAST_OK)
        return rc;
    // the volumes read the offsets just written (same stream): 32-bit intervals wherever a source
    // server's tiles allow it, the 64-bit kernel picks up the rest
    const int items = B * p->S;
    hipLaunchKernelGGL(fastk::rd_volumes32, dim3(fastk::rv_grid(items)), dim3(fastk::RV_THREADS32),
                       fastk::rd_volumes_lds_bytes<int>(p->S), stream,
                       reinterpret_cast<const i64*>(traffic), reinterpret_cast<const i64*>(rebalance),
                       stages, reinterpret_cast<const i64*>(stage_bytes),
                       reinterpret_cast<const i64*>(out_stage_offset), num_stages, p->rdNeed, redis,
                       B, p->S, p->G, p->max_stages);
    hipLaunchKernelGGL(fastk::rd_volumes64, dim3((unsigned)(items < 256 ? items : 256)),
                       dim3(fastk::RV_THREADS64), fastk::rd_volumes_lds_bytes<i64>(p->S), stream,
                       reinterpret_cast<const i64*>(traffic), reinterpret_cast<const i64*>(rebalance),
                       stages, reinterpret_cast<const i64*>(stage_bytes),
                       reinterpret_cast<const i64*>(out_stage_offset), num_stages, p->rdNeed, redis,
                       B, p->S, p->G, p->max_stages);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_redistribution_matrices(fast_plan_t* p, int B, const int64_t* traffic,
                                 const int64_t* rebalance, const int32_t* stages,
                                 const int64_t* stage_bytes, const int32_t* num_stages,
                                 const int64_t* stage_offset, int n_sel, const int32_t* sel,
                                 int64_t* out_matrices, hipStream_t stream) {
    if (!p || B < 0 || n_sel < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0 || n_sel == 0) return FAST_OK;
    if (!traffic || !rebalance || !stages || !stage_bytes || !num_stages || !stage_offset || !sel ||
        !out_matrices)
        return FAST_ERR_INVALID_ARG;
    if (n_sel > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;     // grid.y limit
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    const size_t n = (size_t)n_sel * p->S * p->G * p->G;
    hipLaunchKernelGGL(fastk::rd_zero, dim3((unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256
                                                                            : 2048)),
                       dim3(256), 0, stream, reinterpret_cast<fastk::u64*>(out_matrices), n);
    hipLaunchKernelGGL(fastk::rd_matrices, dim3(p->S, n_sel), dim3(64), 0, stream,
                       reinterpret_cast<const i64*>(traffic), reinterpret_cast<const i64*>(rebalance),
                       stages, reinterpret_cast<const i64*>(stage_bytes),
                       reinterpret_cast<const i64*>(stage_offset), num_stages, sel,
                       reinterpret_cast<i64*>(out_matrices), B, p->S, p->G, p->max_stages);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_plan_summary_batched(fast_plan_t* p, int B, int64_t* out_stage_weight,
                              int64_t* out_scaleup_bytes, hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!out_stage_weight || !out_scaleup_bytes) return FAST_ERR_INVALID_ARG;
    if (B != p->last_B) return FAST_ERR_INVALID_ARG;    // no synthesis call of this size to summarise
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    const int blocks = (p->max_stages + fastk::PL_THREADS - 1) / fastk::PL_THREADS + 1;
    hipLaunchKernelGGL(fastk::pl_summary, dim3(blocks, B), dim3(fastk::PL_THREADS), 0, stream,
                       p->wsPart, p->wsC, reinterpret_cast<i64*>(out_stage_weight),
                       reinterpret_cast<i64*>(out_scaleup_bytes), p->S, p->max_stages);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_pipeline_time_batched(fast_plan_t* p, int B, const int64_t* stage_weight,
                               const int64_t* scaleup_bytes, const int32_t* num_stages,
                               const int32_t* stage_order, const int64_t* redis_bytes,
                               double* out_pipeline_time, hipStream_t stream) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (!stage_weight || !scaleup_bytes || !num_stages || !out_pipeline_time)
        return FAST_ERR_INVALID_ARG;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    hipLaunchKernelGGL(fastk::pl_time, dim3(B), dim3(fastk::PL_THREADS), 0, stream,
                       reinterpret_cast<const i64*>(stage_weight),
                       reinterpret_cast<const i64*>(scaleup_bytes), num_stages, stage_order,
                       reinterpret_cast<const i64*>(redis_bytes), out_pipeline_time, p->G,
                       p->max_stages, p->bw_up, p->bw_out, p->delay);
    if (hipGetLastError() != hipSuccess) return FAST_ERR_HIP;
    return FAST_OK;
}

int fast_plan_set_timing(fast_plan_t* p, int enable) {
    if (!p) return FAST_ERR_INVALID_ARG;
    p->timing = enable ? 1 : 0;
    if (enable) p->n_timed = 0;
    return FAST_OK;
}

int fast_plan_timed_calls(const fast_plan_t* p) { return p ? p->n_timed : -1; }

int fast_plan_kernel_ms(fast_plan_t* p, int call, float* out_ms) {
    if (!p || !out_ms || call < 0 || call >= p->n_timed) return FAST_ERR_INVALID_ARG;
    hipEvent_t* ev = p->ev[call];
    if (hipEventSynchronize(ev[3]) != hipSuccess) {
        (void)hipGetLastError();
        return FAST_ERR_HIP;
    }
    for (int k = 0; k < 3; ++k)
        if (hipEventElapsedTime(&out_ms[k], ev[k], ev[k + 1]) != hipSuccess) {
            (void)hipGetLastError();
            return FAST_ERR_HIP;
        }
    return FAST_OK;
}

int fast_plan_reserve(fast_plan_t* p, int B) {
    if (!p || B < 0) return FAST_ERR_INVALID_ARG;
    if (B == 0) return FAST_OK;
    if (B > FAST_MAX_BATCH) return FAST_ERR_UNSUPPORTED;
    if (const int rc = check_device(p); rc != FAST_OK) return rc;
    int rc = grow_workspace(p, B);
    if (rc == FAST_OK) rc = grow_spo_workspace(p, B);
    if (rc == FAST_OK) rc = grow_so_workspace(p, B);
    if (rc == FAST_OK) rc = grow_rd_workspace(p, B);
    if (rc == FAST_OK) {
        // the chunk totals are the one part whose size does not grow with the batch (small
        // batches are cut into more chunks): b matrices in C chunks need b * (C - 1) tables per
        // block of 64 source servers, which is below 512 / blocks tables and at most 15 * b
        const size_t blocks = (size_t)((p->S + fastk::RD_ROWS - 1) / fastk::RD_ROWS);
        size_t units = (size_t)15 * B * blocks;
        if (units > 512) units = 512;
        rc = grow_chunk_workspace(p, units);
    }
    return rc;
}

void fast_plan_destroy(fast_plan_t* p) {
    if (!p) return;
    free_workspace(p);
    free_spo_workspace(p);
    if (p->soKeys) (void)hipFree(p->soKeys);
    if (p->rdNeed) (void)hipFree(p->rdNeed);
    if (p->rdChunk) (void)hipFree(p->rdChunk);
    if (p->ev) {
        for (int c = 0; c < FAST_MAX_TIMED_CALLS; ++c)
            for (int k = 0; k < 4; ++k)
                if (p->ev[c][k]) (void)hipEventDestroy(p->ev[c][k]);
        delete[] p->ev;
    }
    delete p;
}

}  // extern "C"
