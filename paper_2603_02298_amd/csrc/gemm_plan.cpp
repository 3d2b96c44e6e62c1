#include "gemm_plan.hpp"

#include <algorithm>
#include <cstdlib>

#include "plan.hpp"

namespace lc {

namespace {

// one top-level mode, coalesced (Sec. 3.2), as the kernel's argument
lc_status_t fill_mode(const Modes& m, GemmMode* out) {
  if (m.empty() || (int)m.size() > kGemmMaxLeaves) return LC_ERR_TOO_LARGE;
  out->n = (int32_t)m.size();
  for (const Mode& x : m)
    if (x.extent >= (int64_t(1) << 31) || x.stride >= (int64_t(1) << 31)) return LC_ERR_TOO_LARGE;
  for (int k = 0; k < kGemmMaxLeaves - 1; ++k) {
    const bool reduced = k + 1 < (int)m.size();
    out->div[k] = make_fastdiv(reduced ? (uint32_t)m[k].extent : 1u);
    out->stride[k] = reduced ? (uint32_t)m[k].stride : 0u;
  }
  out->last_stride = (uint32_t)m.back().stride;
  out->lead_stride = (uint32_t)m.front().stride;
  return LC_OK;
}

// Does the mode lead with a stride-1 leaf whose extent is a multiple of `vec`?  Then `vec` consecutive
// coordinates starting at a multiple of `vec` are consecutive in memory.
bool leads_contiguous(const Modes& m, int64_t vec) { return m[0].stride == 1 && m[0].extent % vec == 0; }
// every stride except that of the leading leaf of `lead` is a multiple of `vec` (alignment of every vector)
bool strides_aligned(const Modes& lead, const Modes& other, int64_t vec) {
  for (size_t k = 1; k < lead.size(); ++k)
    if (lead[k].stride % vec != 0) return false;
  for (const Mode& x : other)
    if (x.stride % vec != 0) return false;
  return true;
}

int classify_operand(const Modes& row, const Modes& k, const Modes& batch, unsigned align_bytes) {
  auto plus_batch = [&](Modes other) {
    other.insert(other.end(), batch.begin(), batch.end());
    return other;
  };
  if (align_bytes % 16 == 0) {
    if (leads_contiguous(k, 8) && strides_aligned(k, plus_batch(row), 8)) return kLoadKVec;
    // vectors along the row mode, eight of them (k .. k + 7) per block: k must step evenly inside a block
    if (leads_contiguous(row, 8) && strides_aligned(row, plus_batch(k), 8) && k[0].extent % 8 == 0) return kLoadRVec;
  }
  return kLoadElem;
}

std::string mode_text(const Modes& m) { return Layout::flat(m).str(); }

int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  return (v && *v) ? std::atoi(v) : dflt;
}

}  // namespace

lc_status_t mfma_fragment_layout(int which, Layout* out) {
  if (which == 0 || which == 1) {
    *out = Layout::tuple({Layout::flat({{32, 1}, {2, 256}}), Layout::leaf(8, 32)});
    return LC_OK;
  }
  if (which == 2) {
    *out = Layout::tuple({Layout::flat({{32, 32}, {2, 4}}), Layout::flat({{4, 1}, {4, 8}})});
    return LC_OK;
  }
  return LC_ERR_INVALID_ARG;
}

lc_status_t make_gemm_plan(const Layout& A_in, const Layout& B_in, const Layout& C_in, int ab_dtype, unsigned a_align,
                           unsigned b_align, unsigned c_align, lc_gemm_plan* out) {
  if (ab_dtype != LC_BF16 && ab_dtype != LC_F16) return LC_ERR_UNSUPPORTED_DTYPE;
  for (const Layout* L : {&A_in, &B_in, &C_in}) {
    lc_status_t st = validate(*L);
    if (st != LC_OK) return st;
    // matrices: shapes of rank 2 (Sec. 2.6.2); or all three of rank 3: the batched form of Sec. 1
    if (L->is_leaf() || (L->rank() != 2 && L->rank() != 3) || L->rank() != A_in.rank()) return LC_ERR_INVALID_ARG;
  }
  // preconditions of Sec. 2.6.2
  const int64_t M = A_in.mode(0).size(), K = A_in.mode(1).size(), N = B_in.mode(0).size();
  if (M != C_in.mode(0).size() || N != C_in.mode(1).size() || K != B_in.mode(1).size()) return LC_ERR_SIZE_MISMATCH;
  const bool batched = A_in.rank() == 3;
  const int64_t Lb = batched ? A_in.mode(2).size() : 1;
  if (batched && (Lb != B_in.mode(2).size() || Lb != C_in.mode(2).size())) return LC_ERR_SIZE_MISMATCH;
  if (Lb > 65535) return LC_ERR_TOO_LARGE;   // the batch index is the second grid dimension
  lc_gemm_plan plan;
  plan.ab_dtype = ab_dtype;
  plan.M = M;
  plan.N = N;
  plan.K = K;
  plan.L = Lb;
  plan.a_cosize = A_in.cosize();
  plan.b_cosize = B_in.cosize();
  plan.c_cosize = C_in.cosize();
  const int64_t lim = int64_t(1) << 31;
  if (plan.a_cosize >= lim || plan.b_cosize >= lim || plan.c_cosize >= lim || M >= lim || N >= lim || K >= lim) return LC_ERR_TOO_LARGE;

  // every mode coalesced on its own (Sec. 3.2, by-mode): the kernel evaluates L(r,k) = L_0(r) + L_1(k)
  Modes a_r = coalesce_modes(A_in.mode(0).leaves), a_k = coalesce_modes(A_in.mode(1).leaves);
  Modes b_r = coalesce_modes(B_in.mode(0).leaves), b_k = coalesce_modes(B_in.mode(1).leaves);
  Modes c_m = coalesce_modes(C_in.mode(0).leaves), c_n = coalesce_modes(C_in.mode(1).leaves);
  const Modes unit = {{1, 0}};
  Modes a_l = batched ? coalesce_modes(A_in.mode(2).leaves) : unit, b_l = batched ? coalesce_modes(B_in.mode(2).leaves) : unit;
  Modes c_l = batched ? coalesce_modes(C_in.mode(2).leaves) : unit;

  // C must not alias: many lanes add into it concurrently
  {
    Modes all = c_m;
    all.insert(all.end(), c_n.begin(), c_n.end());
    all.insert(all.end(), c_l.begin(), c_l.end());
    if (M * N * Lb > 1 && !layout_is_injective(all, M * N * Lb)) return LC_ERR_DST_ALIASES;
  }

  // The MFMA result fragment holds four consecutive rows (m) per lane and column.  When C is
  // contiguous along n instead, the roles are exchanged: C^T(n,m) += B(n,k) A(m,k) is the same GEMM
  // with the operands swapped and C's modes exchanged (Table gemm, row "NTT").
  auto with_batch = [](Modes other, const Modes& batch) {
    other.insert(other.end(), batch.begin(), batch.end());
    return other;
  };
  auto c_vec_ok = [&](const Modes& lead, const Modes& other) {
    return c_align % 16 == 0 && leads_contiguous(lead, 4) && strides_aligned(lead, with_batch(other, c_l), 4);
  };
  bool exchange = !c_vec_ok(c_m, c_n) && c_vec_ok(c_n, c_m);
  if (env_int("LC_TUNE_GEMM_EXCHANGE", -1) >= 0) exchange = env_int("LC_TUNE_GEMM_EXCHANGE", 0) != 0;
  unsigned ka_align = a_align, kb_align = b_align;
  if (exchange) {
    std::swap(a_r, b_r);
    std::swap(a_k, b_k);
    std::swap(a_l, b_l);
    std::swap(c_m, c_n);
    std::swap(ka_align, kb_align);
  }
  plan.exchanged = exchange;
  const int64_t kM = exchange ? N : M, kN = exchange ? M : N;

  GemmParams& P = plan.params;
  lc_status_t st;
  if ((st = fill_mode(a_r, &P.a_r)) != LC_OK || (st = fill_mode(a_k, &P.a_k)) != LC_OK || (st = fill_mode(b_r, &P.b_r)) != LC_OK ||
      (st = fill_mode(b_k, &P.b_k)) != LC_OK || (st = fill_mode(c_m, &P.c_m)) != LC_OK || (st = fill_mode(c_n, &P.c_n)) != LC_OK ||
      (st = fill_mode(a_l, &P.a_l)) != LC_OK || (st = fill_mode(b_l, &P.b_l)) != LC_OK || (st = fill_mode(c_l, &P.c_l)) != LC_OK)
    return st;
  P.M = (uint32_t)kM;
  P.N = (uint32_t)kN;
  P.K = (uint32_t)K;
  P.L = (uint32_t)Lb;
  P.a_load = classify_operand(a_r, a_k, a_l, ka_align);
  P.b_load = classify_operand(b_r, b_k, b_l, kb_align);
  const int force = env_int("LC_TUNE_GEMM_LOAD", -1);   // tests: force the element-wise loads
  // element loads are compiled for both operands together: one operand that needs them takes the other along
  if (force == kLoadElem || P.a_load == kLoadElem || P.b_load == kLoadElem) P.a_load = P.b_load = kLoadElem;
  // straight into LDS: k tiles that are contiguous along k
  // (for row vectors: each of the tile's 64 k rows one even step of the k mode's first leaf from the tile's first);
  // compiled for pairs of operands that both qualify
  // A k mode of a single leaf may end in a short k tile: the lanes whose piece lies past K are answered with zeros
  // (k vectors: K a multiple of 8, so that no vector straddles K).
  auto direct_ok = [&](int load, const Modes& k) {
    if (load == kLoadElem) return false;
    if (K % kGemmBK == 0 && k[0].extent % kGemmBK == 0) return true;
    return k.size() == 1 && (load == kLoadRVec || K % 8 == 0) && env_int("LC_TUNE_GEMM_KTAIL", 1) != 0;
  };
  const int direct_env = env_int("LC_TUNE_GEMM_DIRECT", 3);   // bit 0: k vectors, bit 1: row vectors
  auto direct_on = [&](int load) { return (direct_env & (load == kLoadKVec ? 1 : 2)) != 0; };
  const bool direct = direct_ok(P.a_load, a_k) && direct_ok(P.b_load, b_k) && direct_on(P.a_load) && direct_on(P.b_load);
  P.a_direct = P.b_direct = direct ? 1 : 0;
  P.c_vec = c_vec_ok(c_m, c_n) ? 1 : 0;
  if (env_int("LC_TUNE_GEMM_CVEC", 1) == 0) P.c_vec = 0;
  unsigned need_a = P.a_load == kLoadElem ? 2u : 16u, need_b = P.b_load == kLoadElem ? 2u : 16u;
  plan.a_align = exchange ? need_b : need_a;
  plan.b_align = exchange ? need_a : need_b;
  plan.c_align = P.c_vec ? 16u : 4u;

  // tile: 256 x 256 when that still gives every CU a tile, else 128 x 128
  int tile = ((kM + 255) / 256) * ((kN + 255) / 256) * Lb >= 256 ? 256 : 128;
  const int t_env = env_int("LC_TUNE_GEMM_TILE", 0);
  if (t_env == 128 || t_env == 256) tile = t_env;
  plan.tile_m = plan.tile_n = tile;
  P.tiles_m = (uint32_t)((kM + tile - 1) / tile);
  P.tiles_n = (uint32_t)((kN + tile - 1) / tile);
  P.k_tiles = (uint32_t)((K + kGemmBK - 1) / kGemmBK);
  if ((uint64_t)P.tiles_m * P.tiles_n >= (uint64_t(1) << 31)) return LC_ERR_TOO_LARGE;
  P.group_m = (uint32_t)std::max(1, env_int("LC_TUNE_GEMM_GROUP_M", 8));
  // two stages of (rows x 128 bytes) for A and B; direct loads: a ring of five operand tiles
  plan.lds_bytes = direct ? 5u * (unsigned)plan.tile_m * 128u : 2u * (unsigned)(plan.tile_m + plan.tile_n) * 128u;
  plan.a_text = mode_text(a_r) + " x " + mode_text(a_k);
  plan.b_text = mode_text(b_r) + " x " + mode_text(b_k);
  plan.c_text = mode_text(c_m) + " x " + mode_text(c_n);
  if (batched) {
    plan.a_text += " x " + mode_text(a_l);
    plan.b_text += " x " + mode_text(b_l);
    plan.c_text += " x " + mode_text(c_l);
  }
  *out = plan;
  return LC_OK;
}

std::string describe(const lc_gemm_plan& plan) {
  static const char* load_name[] = {"k-vectors", "row-vectors+transpose", "elements"};
  std::string s = "class=gemm-mfma32x32x16 ab=";
  s += plan.ab_dtype == LC_BF16 ? "bf16" : "f16";
  s += " c=f32 M=" + std::to_string(plan.M) + " N=" + std::to_string(plan.N) + " K=" + std::to_string(plan.K);
  if (plan.L != 1 || plan.a_text.find(" x ", plan.a_text.find(" x ") + 1) != std::string::npos) s += " L=" + std::to_string(plan.L);
  s += " exchanged=" + std::to_string((int)plan.exchanged);
  s += " tile=" + std::to_string(plan.tile_m) + "x" + std::to_string(plan.tile_n) + "x" + std::to_string(kGemmBK);
  s += " tiles=" + std::to_string(plan.params.tiles_m) + "x" + std::to_string(plan.params.tiles_n) + " k_tiles=" + std::to_string(plan.params.k_tiles);
  s += " group_m=" + std::to_string(plan.params.group_m);
  s += std::string(" a_load=") + load_name[plan.params.a_load] + (plan.params.a_direct ? "(direct-to-LDS)" : "");
  s += std::string(" b_load=") + load_name[plan.params.b_load] + (plan.params.b_direct ? "(direct-to-LDS)" : "");
  s += " c_vec=" + std::to_string(plan.params.c_vec) + " lds_bytes=" + std::to_string(plan.lds_bytes);
  s += " A=[" + plan.a_text + "] B=[" + plan.b_text + "] C=[" + plan.c_text + "]";
  return s;
}

}  // namespace lc
