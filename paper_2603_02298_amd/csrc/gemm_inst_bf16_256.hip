// Instantiates the generic GEMM kernels for bf16 operands and 256 x 256 tiles.
#include "gemm_kernel.hpp"

namespace lc {
// every pair of load kinds the launcher can ask for (0 k-vectors, 1 row-vectors, 2 elements; 3 and 4: k-vectors and row-vectors
// straight into LDS), instantiated explicitly: left to implicit instantiation through the launcher's chain of templates,
// some pairs stay undefined
template __global__ void gemm_kernel<true, 4, 4, 0, 0>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 0, 1>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 1, 0>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 1, 1>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 3, 3>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 3, 3, true>(GemmParams, const uint16_t*, const uint16_t*, float*);   // K with a short last k tile
template __global__ void gemm_kernel<true, 4, 4, 3, 4>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 3, 4, true>(GemmParams, const uint16_t*, const uint16_t*, float*);   // K with a short last k tile
template __global__ void gemm_kernel<true, 4, 4, 4, 3>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 4, 3, true>(GemmParams, const uint16_t*, const uint16_t*, float*);   // K with a short last k tile
template __global__ void gemm_kernel<true, 4, 4, 4, 4>(GemmParams, const uint16_t*, const uint16_t*, float*);
template __global__ void gemm_kernel<true, 4, 4, 4, 4, true>(GemmParams, const uint16_t*, const uint16_t*, float*);   // K with a short last k tile
template __global__ void gemm_kernel<true, 4, 4, 2, 2>(GemmParams, const uint16_t*, const uint16_t*, float*);

hipError_t launch_gemm_bf16_256(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s) {
  return launch_gemm<true, 4>(plan, a, b, c, s);
}
}  // namespace lc
