// extern "C" boundary of the generic GEMM (include/layoutcopy.h): argument checks and marshalling only.
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>

#include "gemm_plan.hpp"
#include "layoutcopy.h"
#include "plan_cache.hpp"

namespace {
lc_status_t put_text(const std::string& s, char* buf, size_t cap, size_t* needed) {
  if (needed) *needed = s.size() + 1;
  if (buf && cap > 0) {
    size_t n = s.size() < cap - 1 ? s.size() : cap - 1;
    std::memcpy(buf, s.data(), n);
    buf[n] = 0;
  }
  return LC_OK;
}
unsigned pointer_alignment(const void* p) {
  uintptr_t v = reinterpret_cast<uintptr_t>(p);
  unsigned a = 1;
  while (a < 256 && (v % (2 * a)) == 0) a *= 2;
  return a;
}
}  // namespace

extern "C" {

lc_status_t lc_gemm_plan_create(const lc_layout_t* a, const lc_layout_t* b, const lc_layout_t* c, lc_dtype_t ab_dtype, unsigned a_align_bytes,
                                unsigned b_align_bytes, unsigned c_align_bytes, lc_gemm_plan_t** out) {
  if (!a || !b || !c || !out) return LC_ERR_INVALID_ARG;
  if (a->L.has_negative_stride() || b->L.has_negative_stride() || c->L.has_negative_stride()) return LC_ERR_NEGATIVE_STRIDE;   // the GEMM planner's buffer loads take offsets >= 0
  try {
    lc_gemm_plan* p = new lc_gemm_plan;
    lc_status_t st = lc::make_gemm_plan(a->L, b->L, c->L, (int)ab_dtype, a_align_bytes, b_align_bytes, c_align_bytes, p);
    if (st != LC_OK) {
      delete p;
      return st;
    }
    *out = p;
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
void lc_gemm_plan_destroy(lc_gemm_plan_t* plan) { delete plan; }
lc_status_t lc_gemm_plan_describe(const lc_gemm_plan_t* plan, char* buf, size_t cap, size_t* needed) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return put_text(lc::describe(*plan), buf, cap, needed);
}
int64_t lc_gemm_plan_flops(const lc_gemm_plan_t* plan) { return plan ? 2 * plan->M * plan->N * plan->K * plan->L : -1; }
lc_status_t lc_gemm_plan_execute(const lc_gemm_plan_t* plan, const void* a, const void* b, void* c, void* hip_stream) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return lc::execute_gemm_plan(*plan, a, b, c, hip_stream);
}
lc_status_t lc_gemm(const void* a, const lc_layout_t* a_layout, const void* b, const lc_layout_t* b_layout, void* c,
                    const lc_layout_t* c_layout, lc_dtype_t ab_dtype, void* hip_stream) {
  if (!a || !b || !c || !a_layout || !b_layout || !c_layout) return LC_ERR_INVALID_ARG;
  try {
    // plans of recent calls are kept (see plan_cache.hpp); the planner's tuning knobs are part of the key
    std::string key = a_layout->L.str() + "|" + b_layout->L.str() + "|" + c_layout->L.str() + "|" + std::to_string((int)ab_dtype) + "|" +
                      std::to_string(pointer_alignment(a)) + "|" + std::to_string(pointer_alignment(b)) + "|" + std::to_string(pointer_alignment(c));
    for (const char* knob : {"LC_TUNE_GEMM_LOAD", "LC_TUNE_GEMM_DIRECT", "LC_TUNE_GEMM_CVEC", "LC_TUNE_GEMM_TILE", "LC_TUNE_GEMM_GROUP_M",
                             "LC_TUNE_GEMM_EXCHANGE", "LC_TUNE_GEMM_KTAIL"}) {
      const char* v = std::getenv(knob);
      key += std::string(",") + (v ? v : "");
    }
    static lc::PlanCache<lc_gemm_plan> plans;
    std::shared_ptr<const lc_gemm_plan> plan = plans.find(key);
    if (!plan) {
      auto fresh = std::make_shared<lc_gemm_plan>();
      lc_status_t st = lc::make_gemm_plan(a_layout->L, b_layout->L, c_layout->L, (int)ab_dtype, pointer_alignment(a), pointer_alignment(b),
                                          pointer_alignment(c), fresh.get());
      if (st != LC_OK) return st;
      plan = fresh;
      plans.insert(key, plan);
    }
    return lc::execute_gemm_plan(*plan, a, b, c, hip_stream);
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
lc_status_t lc_gemm_plan_time(const lc_gemm_plan_t* plan, const void* a, const void* b, void* c, int warmup, int iters, void* hip_stream,
                              float* ms_per_iter) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return lc::time_gemm_plan(*plan, a, b, c, warmup, iters, hip_stream, ms_per_iter);
}
lc_status_t lc_mfma_fragment_layout(int which, lc_layout_t** out) {
  if (!out) return LC_ERR_INVALID_ARG;
  try {
    lc::Layout L;
    lc_status_t st = lc::mfma_fragment_layout(which, &L);
    if (st != LC_OK) return st;
    *out = new lc_layout_t{L};
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

// Checking device for tests: walks the plan on HOST buffers (see gemm_plan.hpp).  Not in the public header.
lc_status_t lc_debug_gemm_replay_on_host(const lc_gemm_plan_t* plan, const uint16_t* a, int64_t a_elems, const uint16_t* b, int64_t b_elems,
                                         float* c, int64_t c_elems) {
  if (!plan) return LC_ERR_INVALID_ARG;
  try {
    return lc::gemm_replay_on_host(*plan, a, a_elems, b, b_elems, c, c_elems);
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

// Test instrumentation: the kernels' LDS address functions (gemm_params.hpp), so that tests can compare them with
// XOR-stride layouts (Sec. 2.3.2) and model the banks.  what = 0: byte offset of k vector `b` of row `a` in a row-major
// tile; 1: of element (k = a, row = b) in a k-major tile of `rows` rows; 2: the address lane `lane` presents to the
// transpose load of fragment rows a .. a + 31, k = b .. b + 3.  Not in the public header.
int64_t lc_debug_gemm_lds_address(int what, uint32_t rows, uint32_t lane, uint32_t a, uint32_t b) {
  if (what == 0) return lc::gemm_lds_offset(a, b);
  if (what == 1) return lc::gemm_rdirect_lds_offset(rows, a, b);
  if (what == 2) return lc::gemm_rdirect_frag_offset(rows, lane, a, b);
  return -1;
}

}  // extern "C"
