// extern "C" boundary of the library (include/layoutcopy.h): argument checks and marshalling only.
#include <cstring>
#include <new>

#include "algebra.hpp"
#include "layoutcopy.h"
#include "plan.hpp"
#include "plan_cache.hpp"
#include "semimodule.hpp"

namespace {

lc::PlanCache<lc_plan_t>& copy_plans() {
  static lc::PlanCache<lc_plan_t> cache;
  return cache;
}

lc_status_t put_string(const std::string& s, char* buf, size_t cap, size_t* needed) {
  if (needed) *needed = s.size() + 1;
  if (buf && cap > 0) {
    size_t n = s.size() < cap - 1 ? s.size() : cap - 1;
    std::memcpy(buf, s.data(), n);
    buf[n] = 0;
  }
  return LC_OK;
}

lc_status_t give(const lc::Layout& L, lc_layout_t** out) {
  lc_layout_t* h = new (std::nothrow) lc_layout_t{L};
  if (!h) return LC_ERR_INVALID_ARG;
  *out = h;
  return LC_OK;
}

typedef lc_status_t (*binary_op)(const lc::Layout&, const lc::Layout&, lc::Layout*);
// composition's divisibility conditions, complement's ordering and the inverses are stated for strides in N (Sec. 3)
#define LC_REFUSE_NEGATIVE(h) do { if ((h)->L.has_negative_stride()) return LC_ERR_NEGATIVE_STRIDE; } while (0)

lc_status_t binary(binary_op op, const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out) {
  if (!a || !b || !out) return LC_ERR_INVALID_ARG;
  LC_REFUSE_NEGATIVE(a);
  LC_REFUSE_NEGATIVE(b);
  try {
    lc::Layout r;
    lc_status_t st = op(a->L, b->L, &r);
    return st == LC_OK ? give(r, out) : st;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

}  // namespace

extern "C" {

const char* lc_status_string(lc_status_t s) {
  switch (s) {
    case LC_OK: return "OK";
    case LC_ERR_INVALID_ARG: return "INVALID_ARG";
    case LC_ERR_PARSE: return "PARSE";
    case LC_ERR_NOT_CONGRUENT: return "NOT_CONGRUENT";
    case LC_ERR_BAD_EXTENT: return "BAD_EXTENT";
    case LC_ERR_NEGATIVE_STRIDE: return "NEGATIVE_STRIDE";
    case LC_ERR_SIZE_MISMATCH: return "SIZE_MISMATCH";
    case LC_ERR_STRIDE_DIVISIBILITY: return "STRIDE_DIVISIBILITY";
    case LC_ERR_SHAPE_DIVISIBILITY: return "SHAPE_DIVISIBILITY";
    case LC_ERR_NOT_SEGREGATED: return "NOT_SEGREGATED";
    case LC_ERR_NOT_INJECTIVE: return "NOT_INJECTIVE";
    case LC_ERR_NOT_SURJECTIVE: return "NOT_SURJECTIVE";
    case LC_ERR_DST_ALIASES: return "DST_ALIASES";
    case LC_ERR_UNSUPPORTED_DTYPE: return "UNSUPPORTED_DTYPE";
    case LC_ERR_TOO_LARGE: return "TOO_LARGE";
    case LC_ERR_MISALIGNED: return "MISALIGNED";
    case LC_ERR_HIP: return "HIP";
    case LC_ERR_NEEDS_WORKSPACE: return "NEEDS_WORKSPACE";
    case LC_ERR_WORKSPACE_TOO_SMALL: return "WORKSPACE_TOO_SMALL";
    case LC_ERR_SCRATCH_LIMIT: return "SCRATCH_LIMIT";
  }
  return "UNKNOWN";
}

const char* lc_last_hip_error(void) { return lc::last_hip_error(); }

int lc_dtype_bytes(lc_dtype_t dt) {
  switch (dt) {
    case LC_F32: case LC_B32: return 4;
    case LC_F16: case LC_BF16: case LC_B16: return 2;
    case LC_B8: return 1;
    case LC_B64: return 8;
    case LC_B128: return 16;
  }
  return 0;
}

lc_status_t lc_layout_parse(const char* text, lc_layout_t** out) {
  if (!text || !out) return LC_ERR_INVALID_ARG;
  try {
    lc::Layout L;
    lc_status_t st = lc::parse(text, &L);
    return st == LC_OK ? give(L, out) : st;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

lc_status_t lc_layout_from_tree(const int64_t* shape_preorder, int n_nodes, const int64_t* leaf_strides, int n_leaves,
                                lc_layout_t** out) {
  if (!shape_preorder || !leaf_strides || !out || n_nodes < 1 || n_leaves < 1) return LC_ERR_INVALID_ARG;
  try {
    lc::Layout L;
    int leaf = 0;
    for (int k = 0; k < n_nodes; ++k) {
      int64_t v = shape_preorder[k];
      if (v < 0) {
        if (-v > 64) return LC_ERR_INVALID_ARG;
        L.profile.push_back((int32_t)-v);
      } else {
        if (leaf >= n_leaves) return LC_ERR_NOT_CONGRUENT;
        L.profile.push_back(0);
        L.leaves.push_back({v, leaf_strides[leaf++]});
      }
    }
    if (leaf != n_leaves) return LC_ERR_NOT_CONGRUENT;
    lc_status_t st = lc::validate(L);
    return st == LC_OK ? give(L, out) : st;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

void lc_layout_destroy(lc_layout_t* layout) { delete layout; }

lc_status_t lc_layout_to_string(const lc_layout_t* layout, char* buf, size_t cap, size_t* needed) {
  if (!layout) return LC_ERR_INVALID_ARG;
  return put_string(layout->L.str(), buf, cap, needed);
}
int64_t lc_layout_size(const lc_layout_t* layout) { return layout ? layout->L.size() : -1; }
int64_t lc_layout_cosize(const lc_layout_t* layout) { return layout ? layout->L.cosize() : -1; }
int64_t lc_layout_min_offset(const lc_layout_t* layout) { return layout ? layout->L.min_offset() : 1; }
int lc_layout_rank(const lc_layout_t* layout) { return layout ? layout->L.rank() : -1; }
int lc_layout_depth(const lc_layout_t* layout) { return layout ? layout->L.depth() : -1; }
int64_t lc_layout_eval(const lc_layout_t* layout, int64_t i) { return (layout && i >= 0) ? layout->L(i) : -1; }

lc_status_t lc_layout_slice(const lc_layout_t* layout, const char* coord, int64_t* offset, lc_layout_t** out) {
  if (!layout || !coord || !offset || !out) return LC_ERR_INVALID_ARG;
  try {
    lc::Layout r;
    int64_t off = 0;
    lc_status_t st = lc::slice(layout->L, coord, &off, &r);
    if (st != LC_OK) return st;
    st = give(r, out);
    if (st == LC_OK) *offset = off;
    return st;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

lc_status_t lc_coalesce(const lc_layout_t* a, lc_layout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  return give(lc::coalesce(a->L), out);
}
lc_status_t lc_coalesce_bymode(const lc_layout_t* a, lc_layout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  return give(lc::coalesce_bymode(a->L), out);
}
lc_status_t lc_right_inverse(const lc_layout_t* a, lc_layout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  LC_REFUSE_NEGATIVE(a);
  return give(lc::right_inverse(a->L), out);
}
lc_status_t lc_left_inverse(const lc_layout_t* a, lc_layout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  LC_REFUSE_NEGATIVE(a);
  lc::Layout r;
  lc_status_t st = lc::left_inverse(a->L, &r);
  return st == LC_OK ? give(r, out) : st;
}
lc_status_t lc_admissible(const lc_layout_t* a, const lc_layout_t* t, int* yes, lc_layout_t** where) {
  if (!a || !t || !yes) return LC_ERR_INVALID_ARG;
  LC_REFUSE_NEGATIVE(a);
  LC_REFUSE_NEGATIVE(t);
  try {
    bool ok = false, has_where = false;
    lc::Layout w;
    lc_status_t st = lc::admissible(a->L, t->L, &ok, &w, &has_where);
    if (st != LC_OK) return st;
    *yes = ok ? 1 : 0;
    if (where) {
      *where = nullptr;
      if (has_where) return give(w, where);
    }
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
lc_status_t lc_logical_product(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out) { return binary(lc::logical_product, a, b, out); }
lc_status_t lc_blocked_product(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out) { return binary(lc::blocked_product, a, b, out); }
lc_status_t lc_raked_product(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out) { return binary(lc::raked_product, a, b, out); }
lc_status_t lc_composition(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out) { return binary(lc::composition, a, b, out); }
lc_status_t lc_composition_bymode(const lc_layout_t* a, const lc_layout_t* t, lc_layout_t** out) { return binary(lc::composition_bymode, a, t, out); }
lc_status_t lc_logical_divide(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out) { return binary(lc::logical_divide, a, b, out); }
lc_status_t lc_logical_divide_bymode(const lc_layout_t* a, const lc_layout_t* t, lc_layout_t** out) { return binary(lc::logical_divide_bymode, a, t, out); }
lc_status_t lc_zipped_divide(const lc_layout_t* a, const lc_layout_t* t, lc_layout_t** out) { return binary(lc::zipped_divide, a, t, out); }

lc_status_t lc_complement(const lc_layout_t* a, int64_t cotarget, lc_layout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  LC_REFUSE_NEGATIVE(a);
  lc::Layout r;
  lc_status_t st = lc::complement(a->L, cotarget, &r);
  return st == LC_OK ? give(r, out) : st;
}
lc_status_t lc_max_common_vector(const lc_layout_t* a, const lc_layout_t* b, int64_t* K) {
  if (!a || !b || !K) return LC_ERR_INVALID_ARG;
  LC_REFUSE_NEGATIVE(a);
  LC_REFUSE_NEGATIVE(b);
  return lc::max_common_vector(a->L, b->L, K);
}

lc_status_t lc_plan_create(const lc_layout_t* src, const lc_layout_t* dst, lc_dtype_t dt, unsigned src_align_bytes,
                           unsigned dst_align_bytes, lc_plan_t** out) {
  if (!src || !dst || !out) return LC_ERR_INVALID_ARG;
  int es = lc_dtype_bytes(dt);
  if (es == 0) return LC_ERR_UNSUPPORTED_DTYPE;
  try {
    lc_plan_t* plan = new lc_plan_t();
    lc_status_t st = lc::make_plan(src->L, dst->L, es, src_align_bytes, dst_align_bytes, lc::tuning_from_env(), plan);
    if (st != LC_OK) { delete plan; return st; }
    *out = plan;
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
lc_status_t lc_plan_describe(const lc_plan_t* plan, char* buf, size_t cap, size_t* needed) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return put_string(lc::describe(*plan), buf, cap, needed);
}
lc_status_t lc_plan_execute(const lc_plan_t* plan, const void* src, void* dst, void* hip_stream) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return lc::execute_plan(*plan, src, dst, hip_stream);
}
int64_t lc_plan_workspace_bytes(const lc_plan_t* plan) { return plan ? plan->workspace_bytes : -1; }
lc_status_t lc_plan_execute_workspace(const lc_plan_t* plan, const void* src, void* dst, void* workspace, size_t workspace_bytes,
                                      void* hip_stream) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return lc::execute_plan_workspace(*plan, src, dst, workspace, workspace_bytes, hip_stream);
}
size_t lc_static_scratch_bytes(void) { return lc::static_scratch_bytes(); }
lc_status_t lc_plan_execute_static(const lc_plan_t* plan, const void* src, void* dst, void* hip_stream) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return lc::execute_plan_static(*plan, src, dst, hip_stream);
}
void lc_plan_destroy(lc_plan_t* plan) { delete plan; }

lc_status_t lc_copy(const void* src, const lc_layout_t* src_layout, void* dst, const lc_layout_t* dst_layout, lc_dtype_t dt,
                    void* hip_stream) {
  if (!src || !dst || !src_layout || !dst_layout) return LC_ERR_INVALID_ARG;
  auto align_of = [](const void* p) {
    uintptr_t v = reinterpret_cast<uintptr_t>(p);
    unsigned a = 1;
    while (a < 256 && (v % (2 * a)) == 0) a *= 2;
    return a;
  };
  int es = lc_dtype_bytes(dt);
  if (es == 0) return LC_ERR_UNSUPPORTED_DTYPE;
  if (align_of(src) < (unsigned)es || align_of(dst) < (unsigned)es) return LC_ERR_MISALIGNED;
  try {
    // plans of recent calls are kept: planning is host work of some 10 us, several times a short kernel
    const lc::Tuning tune = lc::tuning_from_env();
    std::string key = src_layout->L.str() + "|" + dst_layout->L.str() + "|" + std::to_string(es) + "|" + std::to_string(align_of(src)) + "|" +
                      std::to_string(align_of(dst));
    for (int64_t v : {(int64_t)tune.micro_per_thread, (int64_t)tune.rest_order, (int64_t)tune.wgs_per_cu, (int64_t)tune.unroll,
                      (int64_t)tune.swizzle_shift, (int64_t)tune.nontemporal, (int64_t)tune.blocked, tune.max_items, (int64_t)tune.force_class,
                      (int64_t)tune.max_vec_bytes, (int64_t)tune.tile_queue, (int64_t)tune.queue_rounds, (int64_t)tune.queue_counters,
                      (int64_t)tune.leftover_lead, (int64_t)tune.grid, (int64_t)tune.early_loads, (int64_t)tune.gather, (int64_t)tune.direct_queue})
      key += "," + std::to_string(v);
    for (int64_t v : tune.tile) key += ";" + std::to_string(v);
    std::shared_ptr<const lc_plan_t> plan = copy_plans().find(key);
    if (!plan) {
      auto fresh = std::make_shared<lc_plan_t>();
      lc_status_t st = lc::make_plan(src_layout->L, dst_layout->L, es, align_of(src), align_of(dst), tune, fresh.get());
      if (st != LC_OK) return st;
      plan = fresh;
      copy_plans().insert(key, plan);
    }
    return lc::execute_plan(*plan, src, dst, hip_stream);
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

int64_t lc_plan_algorithmic_bytes(const lc_plan_t* plan) { return plan ? (plan->distinct_reads + plan->n_elems) * plan->elem_bytes : -1; }

lc_status_t lc_plan_time(const lc_plan_t* plan, const void* const* srcs, void* const* dsts, int n_buffers, int warmup, int iters,
                         void* hip_stream, float* ms_per_iter) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return lc::time_plan(*plan, srcs, dsts, n_buffers, warmup, iters, hip_stream, ms_per_iter);
}

lc_status_t lc_plan_time_each(const lc_plan_t* plan, const void* const* srcs, void* const* dsts, int n_buffers, int warmup, int iters,
                              void* hip_stream, float* ms_each) {
  if (!plan) return LC_ERR_INVALID_ARG;
  return lc::time_plan_each(*plan, srcs, dsts, n_buffers, warmup, iters, hip_stream, ms_each);
}

// Checking device for tests: replays the plan's index arithmetic on HOST buffers (see plan.hpp).
// Not declared in the public header; never used to execute a copy.
lc_status_t lc_debug_replay_on_host(const lc_plan_t* plan, const void* src_host, int64_t src_elems, void* dst_host,
                                    int64_t dst_elems, int64_t* lds_conflicts) {
  if (!plan || !src_host || !dst_host) return LC_ERR_INVALID_ARG;
  return lc::replay_on_host(*plan, src_host, 0, src_elems, dst_host, 0, dst_elems, lds_conflicts);
}
// The LDS bank model the planner checks its slot layouts with (test instrumentation): extra cycles of one wavefront
// instruction whose lane l accesses `access_bytes` bytes at byte_addr[l].
int lc_debug_lds_conflicts(const uint32_t* byte_addr_64, int access_bytes, int is_write) {
  bool active[64];
  for (int l = 0; l < 64; ++l) active[l] = true;
  return lc::lds_pass_conflicts(byte_addr_64, active, 64, access_bytes, is_write != 0);
}
// The same for layouts with negative strides: the buffers start src_origin / dst_origin elements before offset 0.
lc_status_t lc_debug_replay_on_host_at(const lc_plan_t* plan, const void* src_buffer, int64_t src_elems, int64_t src_origin, void* dst_buffer,
                                       int64_t dst_elems, int64_t dst_origin, int64_t* lds_conflicts) {
  if (!plan || !src_buffer || !dst_buffer || src_origin < 0 || dst_origin < 0 || src_origin >= src_elems || dst_origin >= dst_elems)
    return LC_ERR_INVALID_ARG;
  const int eb = plan->elem_bytes;
  return lc::replay_on_host(*plan, static_cast<const unsigned char*>(src_buffer) + src_origin * eb, -src_origin, src_elems - src_origin,
                            static_cast<unsigned char*>(dst_buffer) + dst_origin * eb, -dst_origin, dst_elems - dst_origin, lds_conflicts);
}


/* ---- semimodule strides (Sec. 2.3.2) ---- */
lc_status_t lc_slayout_parse(const char* text, lc_slayout_t** out) {
  if (!text || !out) return LC_ERR_INVALID_ARG;
  try {
    lc::SemiLayout L;
    lc_status_t st = lc::parse(text, &L);
    if (st != LC_OK) return st;
    *out = new lc_slayout_t{L};
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
void lc_slayout_destroy(lc_slayout_t* layout) { delete layout; }
lc_status_t lc_slayout_to_string(const lc_slayout_t* layout, char* buf, size_t cap, size_t* needed) {
  if (!layout) return LC_ERR_INVALID_ARG;
  return put_string(layout->L.str(), buf, cap, needed);
}
int lc_slayout_kind(const lc_slayout_t* layout) { return layout ? (int)layout->L.kind() : -1; }
int lc_slayout_codomain_rank(const lc_slayout_t* layout) { return layout ? layout->L.codomain_rank() : -1; }
int64_t lc_slayout_size(const lc_slayout_t* layout) { return layout ? layout->L.size() : -1; }
lc_status_t lc_slayout_eval(const lc_slayout_t* layout, int64_t integral_coord, int64_t* out, int cap) {
  if (!layout || !out || cap < layout->L.codomain_rank()) return LC_ERR_INVALID_ARG;
  layout->L.eval(integral_coord, out);
  return LC_OK;
}
lc_status_t lc_slayout_composition(const lc_slayout_t* a, const lc_layout_t* b, lc_slayout_t** out) {
  if (!a || !b || !out) return LC_ERR_INVALID_ARG;
  try {
    lc::SemiLayout r;
    lc_status_t st = lc::composition(a->L, b->L, &r);
    if (st != LC_OK) return st;
    *out = new lc_slayout_t{r};
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
lc_status_t lc_slayout_coalesce(const lc_slayout_t* a, lc_slayout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  try {
    *out = new lc_slayout_t{lc::coalesce(a->L)};
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
lc_status_t lc_slayout_right_inverse(const lc_slayout_t* a, lc_layout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  try {
    lc::Layout r;
    lc_status_t st = lc::right_inverse(a->L, &r);
    if (st != LC_OK) return st;
    return give(r, out);
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}
lc_status_t lc_slayout_xor_right_inverse(const lc_slayout_t* a, lc_slayout_t** out) {
  if (!a || !out) return LC_ERR_INVALID_ARG;
  try {
    lc::SemiLayout r;
    lc_status_t st = lc::xor_right_inverse(a->L, &r);
    if (st != LC_OK) return st;
    *out = new lc_slayout{r};
    return LC_OK;
  } catch (...) {
    return LC_ERR_INVALID_ARG;
  }
}

}  // extern "C"
