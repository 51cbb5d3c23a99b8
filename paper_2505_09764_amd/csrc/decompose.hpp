// Host-side entry to the two decomposition kernels (k2_birkhoff, k9_bottleneck).  They are
// compiled in a translation unit of their own (decompose.hip) because their stage loops -
// long chains of dependent instructions run by a single wavefront - gain from a scheduling
// strategy of the compiler that the streaming and analysis kernels lose from.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fastk {

// up to this many servers kernel 2 can evaluate the cost model on its own wavefront
constexpr int K2_COST_MAX_S = 32;

// Raises the dynamic-LDS limit of the kernels that serve S servers (above 48 KiB it has to be
// requested per kernel).  Call once per plan.
hipError_t decompose_prepare(int S);

// Embedding + canonical Birkhoff decomposition of B matrices; with_cost (S <= K2_COST_MAX_S
// only): the kernel also writes out_time, otherwise wsT .. delay are not used.
void launch_k2(int S, bool with_cost, int B, hipStream_t stream, const long long* wsQ,
               const long long* wsPart, int32_t* out_stages, long long* out_bytes,
               int32_t* out_num, long long* wsC, int max_stages, const long long* wsT,
               double* out_time, int G, double bw_up, double bw_out, double delay);

// The same with a bottleneck assignment per stage.
void launch_k9(int S, int B, hipStream_t stream, const long long* wsQ, const long long* wsPart,
               int32_t* out_stages, long long* out_bytes, int32_t* out_num, long long* wsC,
               int max_stages);

}  // namespace fastk
