// Seeded synthetic MoE traffic-matrix generator (input data only).
//
// This file holds none of the scheduling method's arithmetic: it only produces
// the int64 GPU-to-GPU byte matrices that the synthesis library and its CPU
// checker are both fed with.  The same sampling routine is compiled for the host
// (fastwl_moe_host) and for the device (fastwl_moe_device) so that a matrix is
// reproducible bit for bit on either side from (seed, b, src, token).
//
// Model: every source GPU routes `tokens` tokens; each token picks `topk`
// distinct experts, drawn one after another from the popularity distribution
// given by `cdf` over popularity ranks (duplicates are redrawn); rank k of matrix
// b lives on GPU gpu_of_rank[b][k]; each pick adds token_bytes to
// traffic[b][src][that GPU].  The GPU diagonal is zeroed at the end.
//
// Random numbers: a counter-based generator, the splitmix64 output function
// applied to a chained key (seed, b, src, token) plus the draw counter.

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__host__ __device__ inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__host__ __device__ inline uint64_t token_key(uint64_t seed, uint32_t b, uint32_t src,
                                              uint32_t token) {
    uint64_t h = mix64(seed);
    h = mix64(h + b);
    h = mix64(h + src);
    h = mix64(h + token);
    return h;
}

constexpr int kMaxTopK = 16;
constexpr uint32_t kMaxDraws = 1u << 16;

// Picks `topk` distinct ranks for one token; writes them to picks[].
__host__ __device__ inline void route_token(uint64_t key, const double* cdf, int E, int topk,
                                            int* picks) {
    int n = 0;
    uint32_t draw = 0;
    while (n < topk) {
        int k;
        if (draw < kMaxDraws) {
            const uint64_t x = mix64(key + draw);
            const double u = (double)(x >> 11) * (1.0 / 9007199254740992.0);
            int lo = 0, hi = E - 1;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (cdf[mid] > u) hi = mid; else lo = mid + 1;
            }
            k = lo;
            ++draw;
            bool dup = false;
            for (int q = 0; q < n; ++q) dup = dup || (picks[q] == k);
            if (dup) continue;
        } else {
            // Draw budget exhausted (practically unreachable): lowest unused rank.
            k = 0;
            for (;;) {
                bool dup = false;
                for (int q = 0; q < n; ++q) dup = dup || (picks[q] == k);
                if (!dup) break;
                ++k;
            }
        }
        picks[n++] = k;
    }
}

__global__ void __launch_bounds__(256)
moe_kernel(int64_t* __restrict__ traffic, const double* __restrict__ cdf,
           const int32_t* __restrict__ gpu_of_rank, int N, int E, int tokens, int topk,
           int64_t token_bytes, uint64_t seed) {
    extern __shared__ unsigned char smem_raw[];
    double* s_cdf = reinterpret_cast<double*>(smem_raw);
    uint32_t* s_cnt = reinterpret_cast<uint32_t*>(s_cdf + E);
    const int src = blockIdx.x;
    const int b = blockIdx.y;
    for (int k = threadIdx.x; k < E; k += blockDim.x) s_cdf[k] = cdf[k];
    for (int h = threadIdx.x; h < N; h += blockDim.x) s_cnt[h] = 0;
    __syncthreads();
    const int32_t* map = gpu_of_rank + (size_t)b * E;
    for (int t = threadIdx.x; t < tokens; t += blockDim.x) {
        int picks[kMaxTopK];
        route_token(token_key(seed, b, src, t), s_cdf, E, topk, picks);
        for (int q = 0; q < topk; ++q) atomicAdd(&s_cnt[map[picks[q]]], 1u);
    }
    __syncthreads();
    int64_t* row = traffic + ((size_t)b * N + src) * N;
    for (int h = threadIdx.x; h < N; h += blockDim.x)
        row[h] = (h == src) ? 0 : (int64_t)s_cnt[h] * token_bytes;
}

bool args_ok(const void* traffic, const void* cdf, const void* map, int B, int N, int E,
             int tokens, int topk) {
    return traffic && cdf && map && B >= 0 && N >= 1 && E >= 1 && tokens >= 0 && topk >= 1 &&
           topk <= kMaxTopK && topk <= E;
}

}  // namespace

extern "C" {

// Host version.  traffic[B][N][N], cdf[E], gpu_of_rank[B][E] are host pointers.
// Matrices [b_begin, b_end) are written (so callers can split a batch over
// threads).  Returns 0, or -1 on bad arguments.
int fastwl_moe_host(int64_t* traffic, const double* cdf, const int32_t* gpu_of_rank, int B, int N,
                    int E, int tokens, int topk, int64_t token_bytes, uint64_t seed, int b_begin,
                    int b_end) {
    if (!args_ok(traffic, cdf, gpu_of_rank, B, N, E, tokens, topk)) return -1;
    if (b_begin < 0 || b_end > B || b_begin > b_end) return -1;
    for (int b = b_begin; b < b_end; ++b) {
        const int32_t* map = gpu_of_rank + (size_t)b * E;
        for (int src = 0; src < N; ++src) {
            int64_t* row = traffic + ((size_t)b * N + src) * N;
            for (int h = 0; h < N; ++h) row[h] = 0;
            for (int t = 0; t < tokens; ++t) {
                int picks[kMaxTopK];
                route_token(token_key(seed, b, src, t), cdf, E, topk, picks);
                for (int q = 0; q < topk; ++q) row[map[picks[q]]] += token_bytes;
            }
            row[src] = 0;
        }
    }
    return 0;
}

// Device version.  All pointers are device memory on the current device; work
// is enqueued on `stream` and not synchronised.  Returns 0, -1 on bad
// arguments, -3 if the launch failed.
int fastwl_moe_device(int64_t* traffic, const double* cdf, const int32_t* gpu_of_rank, int B,
                      int N, int E, int tokens, int topk, int64_t token_bytes, uint64_t seed,
                      hipStream_t stream) {
    if (!args_ok(traffic, cdf, gpu_of_rank, B, N, E, tokens, topk)) return -1;
    if (B == 0) return 0;
    if (B > 65535) return -1;
    const size_t smem = (size_t)E * sizeof(double) + (size_t)N * sizeof(uint32_t);
    if (smem > 60 * 1024) return -1;
    hipLaunchKernelGGL(moe_kernel, dim3(N, B), dim3(256), smem, stream, traffic, cdf, gpu_of_rank,
                       N, E, tokens, topk, token_bytes, seed);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

}  // extern "C"
