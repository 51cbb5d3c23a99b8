// The decomposition kernels and their launchers; see decompose.hpp for why they are built apart.
#include "decompose.hpp"

#include "k2_birkhoff.hpp"
#include "k9_bottleneck.hpp"

namespace fastk {

namespace {

typedef void (*k2_fn)(const i64*, const i64*, int32_t*, i64*, int32_t*, i64*, int, int, const i64*,
                      double*, int, double, double, double);
typedef void (*k9_fn)(const i64*, const i64*, int32_t*, i64*, int32_t*, i64*, int, int);

// One or two rows per lane, the variant without bounds predicates when S fills the wavefront
// exactly, and for small clusters the variant that carries the cost model.
k2_fn k2_kernel(int S, bool with_cost) {
    if (S == 128) return &k2_birkhoff<2, true, false>;
    if (S > 64) return &k2_birkhoff<2, false, false>;
    if (S == 64) return &k2_birkhoff<1, true, false>;
    if (with_cost && S <= K2_COST_MAX_S) return &k2_birkhoff<1, false, true>;
    return &k2_birkhoff<1, false, false>;
}
k9_fn k9_kernel(int S) { return S > 64 ? &k9_bottleneck<2> : &k9_bottleneck<1>; }

}  // namespace

hipError_t decompose_prepare(int S) {
    // The kernels keep the S x S residual in LDS: up to 133 KiB of the CU's 160 KiB.
    hipError_t e = hipSuccess;
    if (k2_lds_bytes(S) > 48 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k2_kernel(S, false)),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)k2_lds_bytes(S));
    if (e == hipSuccess && k9_lds_bytes(S) > 48 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(k9_kernel(S)),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)k9_lds_bytes(S));
    return e;
}

void launch_k2(int S, bool with_cost, int B, hipStream_t stream, const long long* wsQ,
               const long long* wsPart, int32_t* out_stages, long long* out_bytes,
               int32_t* out_num, long long* wsC, int max_stages, const long long* wsT,
               double* out_time, int G, double bw_up, double bw_out, double delay) {
    hipLaunchKernelGGL(k2_kernel(S, with_cost), dim3(B), dim3(K2_THREADS), k2_lds_bytes(S), stream,
                       wsQ, wsPart, out_stages, out_bytes, out_num, wsC, S, max_stages, wsT,
                       out_time, G, bw_up, bw_out, delay);
}

void launch_k9(int S, int B, hipStream_t stream, const long long* wsQ, const long long* wsPart,
               int32_t* out_stages, long long* out_bytes, int32_t* out_num, long long* wsC,
               int max_stages) {
    hipLaunchKernelGGL(k9_kernel(S), dim3(B), dim3(K9_THREADS), k9_lds_bytes(S), stream, wsQ,
                       wsPart, out_stages, out_bytes, out_num, wsC, S, max_stages);
}

}  // namespace fastk
