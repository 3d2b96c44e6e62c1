// Launch side of the generic GEMM: picks the instantiation (element type, tile size) a plan asks for.  The
// kernels live in gemm_kernel.hpp and are instantiated in gemm_inst_*.hip.
#include <hip/hip_runtime.h>

#include <string>

#include "gemm_plan.hpp"
#include "plan.hpp"

namespace lc {

hipError_t launch_gemm_bf16_256(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s);
hipError_t launch_gemm_bf16_128(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s);
hipError_t launch_gemm_f16_256(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s);
hipError_t launch_gemm_f16_128(const lc_gemm_plan& plan, const uint16_t* a, const uint16_t* b, float* c, hipStream_t s);

static bool gemm_hip_failed(hipError_t e, const char* what) {
  if (e == hipSuccess) return false;
  set_last_hip_error(std::string(what) + ": " + hipGetErrorName(e) + " (" + hipGetErrorString(e) + ")");
  return true;
}

lc_status_t execute_gemm_plan(const lc_gemm_plan& plan, const void* a, const void* b, void* c, void* stream) {
  if (!a || !b || !c) return LC_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(a) % plan.a_align || reinterpret_cast<uintptr_t>(b) % plan.b_align ||
      reinterpret_cast<uintptr_t>(c) % plan.c_align)
    return LC_ERR_MISALIGNED;
  // the kernel's A is the operand whose rows run along the kernel's m
  const uint16_t* ka = static_cast<const uint16_t*>(plan.exchanged ? b : a);
  const uint16_t* kb = static_cast<const uint16_t*>(plan.exchanged ? a : b);
  float* kc = static_cast<float*>(c);
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  hipError_t pre;
  const bool bf16 = plan.ab_dtype == LC_BF16;
  // LDS the kernels assume: two stages of an A and a B tile, or (direct loads, always as a pair) a ring of five tiles
  if (plan.params.a_direct != plan.params.b_direct) return LC_ERR_INVALID_ARG;
  const unsigned tiles_in_lds = plan.params.a_direct ? 5u : 4u;
  if (plan.tile_m == 256 && plan.tile_n == 256 && plan.lds_bytes == tiles_in_lds * 256u * 128u)
    pre = bf16 ? launch_gemm_bf16_256(plan, ka, kb, kc, s) : launch_gemm_f16_256(plan, ka, kb, kc, s);
  else if (plan.tile_m == 128 && plan.tile_n == 128 && plan.lds_bytes == tiles_in_lds * 128u * 128u)
    pre = bf16 ? launch_gemm_bf16_128(plan, ka, kb, kc, s) : launch_gemm_f16_128(plan, ka, kb, kc, s);
  else
    return LC_ERR_INVALID_ARG;
  if (gemm_hip_failed(pre, "hipFuncSetAttribute") || gemm_hip_failed(hipGetLastError(), "kernel launch")) return LC_ERR_HIP;
  return LC_OK;
}

lc_status_t time_gemm_plan(const lc_gemm_plan& plan, const void* a, const void* b, void* c, int warmup, int iters, void* stream,
                           float* ms_per_iter) {
  if (iters < 1 || warmup < 0 || !ms_per_iter) return LC_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  if (gemm_hip_failed(hipEventCreate(&e0), "hipEventCreate")) return LC_ERR_HIP;
  if (gemm_hip_failed(hipEventCreate(&e1), "hipEventCreate")) { (void)hipEventDestroy(e0); return LC_ERR_HIP; }
  lc_status_t st = LC_OK;
  for (int i = 0; i < warmup && st == LC_OK; ++i) st = execute_gemm_plan(plan, a, b, c, stream);
  if (st == LC_OK && gemm_hip_failed(hipEventRecord(e0, s), "hipEventRecord")) st = LC_ERR_HIP;
  for (int i = 0; i < iters && st == LC_OK; ++i) st = execute_gemm_plan(plan, a, b, c, stream);
  if (st == LC_OK && gemm_hip_failed(hipEventRecord(e1, s), "hipEventRecord")) st = LC_ERR_HIP;
  if (st == LC_OK && gemm_hip_failed(hipEventSynchronize(e1), "hipEventSynchronize")) st = LC_ERR_HIP;
  float ms = 0.f;
  if (st == LC_OK && gemm_hip_failed(hipEventElapsedTime(&ms, e0, e1), "hipEventElapsedTime")) st = LC_ERR_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st == LC_OK) *ms_per_iter = ms / (float)iters;
  return st;
}

}  // namespace lc
