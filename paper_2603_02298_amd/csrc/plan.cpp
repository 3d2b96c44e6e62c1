#include "plan.hpp"

#include <algorithm>
#include <cstdlib>
#include <cstring>

namespace lc {

static int env_int(const char* name, int dflt) {
  const char* v = std::getenv(name);
  return (v && *v) ? std::atoi(v) : dflt;
}

Tuning tuning_from_env() {
  Tuning t;
  t.micro_per_thread = env_int("LC_TUNE_MICRO_PER_THREAD", t.micro_per_thread);
  t.rest_order = env_int("LC_TUNE_REST_ORDER", t.rest_order);
  t.wgs_per_cu = env_int("LC_TUNE_WGS_PER_CU", t.wgs_per_cu);
  t.unroll = env_int("LC_TUNE_UNROLL", t.unroll);
  t.swizzle_shift = env_int("LC_TUNE_SWIZZLE_SHIFT", t.swizzle_shift);
  t.nontemporal = env_int("LC_TUNE_NONTEMPORAL", t.nontemporal);
  t.force_class = env_int("LC_TUNE_FORCE_CLASS", t.force_class);
  t.max_vec_bytes = env_int("LC_TUNE_MAX_VEC_BYTES", t.max_vec_bytes);
  t.blocked = env_int("LC_TUNE_BLOCKED", t.blocked);
  t.tile_queue = env_int("LC_TUNE_TILE_QUEUE", t.tile_queue);
  t.queue_rounds = env_int("LC_TUNE_QUEUE_ROUNDS", t.queue_rounds);
  t.queue_counters = env_int("LC_TUNE_QUEUE_COUNTERS", t.queue_counters);
  t.leftover_lead = env_int("LC_TUNE_LEFTOVER_LEAD", t.leftover_lead);
  t.grid = env_int("LC_TUNE_GRID", t.grid);
  t.early_loads = env_int("LC_TUNE_EARLY_LOADS", t.early_loads);
  t.gather = env_int("LC_TUNE_GATHER", t.gather);
  t.direct_queue = env_int("LC_TUNE_DIRECT_QUEUE", t.direct_queue);
  t.max_items = env_int("LC_TUNE_MAX_ITEMS", (int)t.max_items);
  if (const char* v = std::getenv("LC_TUNE_TILE")) {
    for (const char* p = v; *p;) {
      t.tile.push_back(std::strtoll(p, const_cast<char**>(&p), 10));
      if (*p == ',') ++p; else break;
    }
  }
  return t;
}

// ---------------------------------------------------------------------------------------------
// a1: is the destination layout injective?  Nested strides prove it; otherwise small layouts are
// enumerated and large ones are refused.
// ---------------------------------------------------------------------------------------------
bool layout_is_injective(const Modes& coalesced, int64_t n) {
  Modes m;
  for (const Mode& x : coalesced) {
    if (x.extent == 1) continue;
    if (x.stride == 0) return false;
    m.push_back(x);
  }
  std::stable_sort(m.begin(), m.end(), [](const Mode& x, const Mode& y) { return x.stride < y.stride; });
  bool nested = true;
  int64_t covered = 1;
  for (const Mode& x : m) {
    if (x.stride < covered) nested = false;
    covered = x.stride * (x.extent - 1) + covered;   // largest offset so far + 1
  }
  if (nested) return true;
  if (n > (1 << 22)) return false;   // cannot be proved cheaply: refuse rather than risk a race
  std::vector<int64_t> offs((size_t)n);
  Layout L = Layout::flat(coalesced);
  for (int64_t i = 0; i < n; ++i) offs[(size_t)i] = L(i);
  std::sort(offs.begin(), offs.end());
  return std::adjacent_find(offs.begin(), offs.end()) == offs.end();
}

// ---------------------------------------------------------------------------------------------
// a3: the coarsest shape that refines both flat shapes (mixed-radix boundaries must nest).
// ---------------------------------------------------------------------------------------------
static bool common_refinement(const Modes& S, const Modes& D, std::vector<int64_t>* F) {
  size_t i = 0, j = 0;
  int64_t x = S[0].extent, y = D[0].extent;
  for (;;) {
    int64_t g = std::min(x, y);
    if (x % g != 0 || y % g != 0) return false;
    F->push_back(g);
    x /= g;
    y /= g;
    if (x == 1) { if (++i < S.size()) x = S[i].extent; }
    if (y == 1) { if (++j < D.size()) y = D[j].extent; }
    if (i == S.size() || j == D.size()) break;
  }
  return i == S.size() && j == D.size();
}

static int pow2_floor(int64_t v) { int p = 1; while (2 * p <= v) p *= 2; return p; }

// Largest power of two <= cap that divides every listed quantity.
static int common_pow2(int cap, const std::vector<int64_t>& must_divide) {
  int v = pow2_floor(cap);
  for (; v > 1; v /= 2) {
    bool ok = true;
    for (int64_t x : must_divide) if (x % v != 0) { ok = false; break; }
    if (ok) break;
  }
  return v;
}

// ---------------------------------------------------------------------------------------------
// LDS bank model (checks the swizzle; reported by the host replay).  Measured on gfx950 with SQ_LDS_BANK_CONFLICT on
// address patterns made for the purpose (one wavefront, per instruction):
//   width   write: lanes per pass, banks repeat every    read: lanes per pass, banks repeat every
//   16 B    8 consecutive lanes,   128 bytes             16 lanes (*),          256 bytes
//    8 B    16 consecutive lanes,  128 bytes             32 consecutive lanes,  256 bytes
//    4 B    32 consecutive lanes,  128 bytes             32 consecutive lanes,  128 bytes
//   (*) in each half of the wavefront the 4-lane groups 0,3,5,6 go together and so do 1,2,4,7 (equal parity of the
//       group index's bits): lanes 0-3,12-15,20-27 and 4-11,16-19,28-31.
// A pass takes as many cycles as the most loaded bank has distinct dwords; cost = cycles beyond one per pass.
// ---------------------------------------------------------------------------------------------
static int lds_pass_of_lane(int lane, int access_bytes, bool is_write) {
  if (is_write) return lane / (128 / std::max(4, std::min(16, access_bytes)));
  if (access_bytes >= 16) {
    const int group = (lane / 4) % 8;
    const int parity = (group ^ (group >> 1) ^ (group >> 2)) & 1;
    return (lane / 32) * 2 + parity;
  }
  return lane / 32;
}
int lds_pass_conflicts(const uint32_t* byte_addr, const bool* active, int lanes, int access_bytes, bool is_write) {
  const int words = access_bytes >= 4 ? access_bytes / 4 : 1;
  const uint32_t banks = (is_write || access_bytes <= 4) ? 32u : 64u;
  int cost = 0;
  for (int pass = 0; pass < 8; ++pass) {
    uint8_t cnt[64];
    uint32_t seen[64][8];
    std::memset(cnt, 0, sizeof(cnt));
    bool any = false;
    for (int l = 0; l < lanes; ++l) {
      if (!active[l] || lds_pass_of_lane(l, access_bytes, is_write) != pass) continue;
      any = true;
      for (int w = 0; w < words; ++w) {
        const uint32_t dword = byte_addr[l] / 4 + (uint32_t)w, bank = dword % banks;
        bool again = false;
        for (int k = 0; k < cnt[bank] && k < 8; ++k) if (seen[bank][k] == dword) again = true;   // the same dword: one access
        if (again) continue;
        if (cnt[bank] < 8) seen[bank][cnt[bank]] = dword;
        cnt[bank]++;
      }
    }
    if (!any) continue;
    int worst = 1;
    for (uint32_t b = 0; b < banks; ++b) worst = std::max<int>(worst, cnt[b]);
    cost += worst - 1;
  }
  return cost;
}

int transpose_swizzle_cost(const TransposeParams& P, int V, int es, uint32_t max_waves, int max_ip, int lanes = 64) {
  // parks: lane u writes vector (u, ip) at slot(g0(u) + ip * gpos_pv); picks: lane reads slot(g) for consecutive g
  int cost = 0;
  int slot_bytes = V * es;
  uint32_t waves = std::min<uint32_t>((P.n_micro + 63) / 64, max_waves);
  for (uint32_t wv = 0; wv < waves; ++wv) {
    uint32_t g0[64];
    bool act[64];
    for (int l = 0; l < 64; ++l) {
      uint32_t u = wv * 64 + (uint32_t)l;
      act[l] = u < P.n_micro;
      int32_t so;
      g0[l] = 0;
      if (act[l]) micro_from_src_order(P, u, &so, &g0[l]);
    }
    for (int ip = 0; ip < V && ip < max_ip; ++ip) {
      uint32_t wa[64];
      for (int l = 0; l < 64; ++l) wa[l] = lds_slot(P, g0[l] + (uint32_t)ip * P.gpos_pv) * (uint32_t)slot_bytes;
      cost += lds_pass_conflicts(wa, act, lanes, slot_bytes, true);
    }
  }
  uint32_t pick_waves = std::min<uint32_t>((P.n_vec + 63) / 64, max_waves);
  for (uint32_t wv = 0; wv < pick_waves; ++wv) {
    uint32_t ra[64];
    bool act[64];
    for (int l = 0; l < 64; ++l) {
      uint32_t g = wv * 64 + (uint32_t)l;
      act[l] = g < P.n_vec;
      ra[l] = lds_slot(P, g) * (uint32_t)slot_bytes;
    }
    cost += lds_pass_conflicts(ra, act, lanes, slot_bytes, false);
  }
  return cost;
}

// Contiguous run length (elements) of a tile along one side: follow the modes in stride order
// (`order`, computed once per plan) starting at stride 1 while each is fully inside the tile and the
// next continues it.
static std::vector<int> stride_order(const std::vector<JointMode>& J, bool src_side) {
  std::vector<int> order;
  for (int k = 0; k < (int)J.size(); ++k) order.push_back(k);
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
    return (src_side ? J[(size_t)x].a : J[(size_t)x].b) < (src_side ? J[(size_t)y].a : J[(size_t)y].b);
  });
  return order;
}
static int64_t run_length(const std::vector<JointMode>& J, const std::vector<int>& order, const std::vector<int64_t>& t,
                          bool src_side) {
  int64_t run = 1, expect = 1;
  for (int k : order) {
    int64_t st = src_side ? J[(size_t)k].a : J[(size_t)k].b;
    if (st <= 0) continue;   // a broadcast or a reversed mode is no part of a contiguous run
    if (st != expect) break;
    run *= t[(size_t)k];
    if (t[(size_t)k] < J[(size_t)k].extent) break;
    expect = st * J[(size_t)k].extent;
  }
  return run;
}

static int64_t smallest_prime_factor(int64_t v) {
  for (int64_t f = 2; f * f <= v; ++f) if (v % f == 0) return f;
  return v;
}

static void fill_flat_arg(const Modes& m, FlatLayoutArg* out) {
  out->n_modes = (int32_t)m.size();
  for (size_t k = 0; k < m.size(); ++k) {
    out->div[k] = make_fastdiv((uint32_t)m[k].extent);
    out->stride[k] = m[k].stride;
  }
}

static lc_status_t plan_generic(const Modes& S, const Modes& D, int64_t n, lc_plan* plan, const std::string& why) {
  if (S.size() > (size_t)kMaxGenericModes || D.size() > (size_t)kMaxGenericModes || n >= (1ll << 31)) return LC_ERR_TOO_LARGE;
  plan->cls = KernelClass::Generic;
  fill_flat_arg(S, &plan->generic.src);
  fill_flat_arg(D, &plan->generic.dst);
  plan->generic.n = (uint32_t)n;
  plan->width_bytes = plan->elem_bytes;
  plan->note = why;
  return LC_OK;
}

// Destinations that alias (Table copy, "Scatter" with repeated offsets; Sec. 2.6.1: the loop's last write stays).
static lc_status_t plan_last_writer(const Modes& S, const Modes& D, int64_t n, lc_plan* plan, const std::string& why) {
  int64_t span = 1, lowest = 0;   // offsets the destination reaches: lowest .. lowest + span - 1
  for (const Mode& m : D) {
    span += (m.extent - 1) * std::abs(m.stride);
    if (m.stride < 0) lowest += (m.extent - 1) * m.stride;
  }
  lc_status_t st = plan_generic(S, D, n, plan, why);
  if (st != LC_OK) return st;
  if (span >= (1ll << 40)) return LC_ERR_TOO_LARGE;
  plan->cls = KernelClass::LastWriter;
  plan->workspace_bytes = span * 4;
  plan->workspace_bias = -lowest;
  plan->wgs_per_cu = 16;
  return LC_OK;
}

static bool transpose_instantiated(int es, int V) {
  return (es == 4 && (V == 4 || V == 2)) || (es == 2 && (V == 8 || V == 4 || V == 2)) || (es == 16 && V == 1);
}
// the ragged kernel also moves single elements (V = 1) of any width
static bool ragged_instantiated(int es, int V) {
  return transpose_instantiated(es, V) || (V == 1 && (es == 1 || es == 2 || es == 4 || es == 8 || es == 16));
}

// The fourteen dwords the first loads of a launch can be computed from (TransposeHead), when the plan fits them.
static void fill_transpose_head(const TransposeParams& P, int micro_per_thread, TransposeHead* H) {
  std::memset(H, 0, sizeof(*H));
  if (micro_per_thread != 1 || P.n_ragged != 0 || P.blocked || P.src_split < 1 || P.src_split > 4 || P.n_rest > 2 || P.n_micro > (uint32_t)kBlock)
    return;
  uint32_t ctl = 1u, taken = 0;
  for (int k = 0; k < P.src_split; ++k) {
    // modes below the last one the lane reaches have extents that divide kBlock (powers of two); the last takes what is left
    uint32_t bits = 8;
    if (k + 1 < P.src_split) {
      bits = 0;
      while ((1u << bits) < P.ext_s[k].div) ++bits;
      if ((1u << bits) != P.ext_s[k].div) return;
    }
    ctl |= bits << (1 + 4 * k);
    taken += bits;
    H->sa[k] = P.sa_s[k];
  }
  if (taken < 8) return;
  // tile id -> (r, q) by the first rest mode; a grid of one mode (or a single tile) divides by more than any tile id
  const FastDiv d = P.n_rest == 2 ? P.rdiv[0] : make_fastdiv(0x7fffffffu);
  H->r0_mul = d.mul;
  H->r0_div = d.div;
  ctl |= (d.shift & 31u) << 17;
  ctl |= P.n_micro << 22;
  H->ra0 = P.n_rest >= 1 ? P.ra[0] : 0;
  H->ra1 = P.n_rest == 2 ? P.ra[1] : 0;
  H->a_q = P.a_q;
  H->ctl = ctl;
  // the head must say what the argument block says: every lane's offset and every tile's origin
  for (uint32_t lane = 0; lane < (uint32_t)kBlock; ++lane) {
    int32_t so;
    uint32_t g0;
    micro_lane_part(P, lane, &so, &g0);
    if (lane < P.n_micro && head_lane_offset(*H, lane) != so + P.src_trip_off[0]) { H->ctl = 0; return; }
  }
  // (a workgroup's first tile is its index in the grid: the launcher uses the head only for grids within kHeadMaxGrid)
  for (uint32_t t = 0; t < std::min<uint32_t>(P.n_tiles, (uint32_t)kHeadMaxGrid); ++t) {
    int64_t so, dof;
    tile_origin(P, t, &so, &dof);
    if (head_tile_origin(*H, t) != so) { H->ctl = 0; return; }
  }
}

// Tiles a copy over joint modes J (extents and strides in units of `es` bytes) for the transposing
// kernel with V x V micro-tiles; p / q are the modes the micro-tile extends along on the source /
// destination side.  Fills the plan and returns true, or leaves the class undecided.
// ragged: tile extents are powers of two (times V along p and q) and need not divide the extents; the
// grid has ceil(extent / tile) tiles along such a mode and the kernel checks coordinates at the edge.
static bool plan_tiled(const std::vector<JointMode>& J, int es, int V, int p, int q, int64_t n, const Tuning& tune, lc_plan* plan,
                       bool ragged = false) {
  const int nj = (int)J.size();
  // Tile size: up to 4 micro-tiles per lane (64 KiB of fp32), but never so large that fewer than
  // ~1024 tiles remain for the 256 CUs; growth stops early once both sides move >= 512-byte runs.
  // 32 KiB of 16-byte words, 64 KiB of 4 x 4 fp32 micro-tiles; single elements: 4 per lane measured best (35 % of
  // the HBM peak on a 4001 x 4003 fp32 transpose against 26 % with 8 and 24 % with 1)
  const int max_per_lane = V == 1 ? (es == 16 ? 8 : 4) : 4;
  int64_t target = (int64_t)max_per_lane * kBlock;
  while (target > 64 && n / (target * V * V) < 1024) target /= 2;
  if (tune.micro_per_thread == 1 || tune.micro_per_thread == 2 || tune.micro_per_thread == 4 || (tune.micro_per_thread == 8 && V == 1))
    target = (int64_t)kBlock * tune.micro_per_thread;
  const int64_t enough_run_bytes = 512;
  // a lane should have about eight 16-byte loads in flight: one V = 8 micro-tile, or eight single words
  const int64_t full_wg = (int64_t)kBlock * (V == 1 ? max_per_lane : 1);
  const std::vector<int> src_order = stride_order(J, true), dst_order = stride_order(J, false);
  // a6: grow the tile one prime factor at a time, always helping the shorter contiguous run
  std::vector<int64_t> t((size_t)nj, 1);
  t[(size_t)p] = V;
  t[(size_t)q] = V;
  int64_t micro = 1;
  // offsets inside a tile are 32-bit in the kernel: a growth step must keep both spans below 2^30 elements
  auto spans_fit = [&](const std::vector<int64_t>& tt) {
    int64_t ss = 0, sd = 0;
    for (int k = 0; k < nj; ++k) { ss += (tt[(size_t)k] - 1) * std::abs(J[(size_t)k].a); sd += (tt[(size_t)k] - 1) * J[(size_t)k].b; }
    return ss < (1ll << 30) && sd < (1ll << 30);
  };
  auto micro_of = [&](const std::vector<int64_t>& tt) {
    int64_t m = 1;
    for (int k = 0; k < nj; ++k) m *= (k == p || k == q) ? (tt[(size_t)k] + V - 1) / V : tt[(size_t)k];
    return m;
  };
  while (ragged) {
    // double the tile along the mode that lengthens the shorter run most; a tile that would reach past
    // the extent takes the whole extent instead (that mode is then not ragged)
    int best = -1;
    int64_t best_min = -1, best_sum = -1, best_t = 1;
    for (int k = 0; k < nj; ++k) {
      const int64_t e = J[(size_t)k].extent, old = t[(size_t)k];
      if (old >= e) continue;
      const int64_t grown = std::min<int64_t>(old * 2, e);
      t[(size_t)k] = grown;
      const bool fits = spans_fit(t) && micro_of(t) <= target && grown < (1 << 15);
      int64_t rs = run_length(J, src_order, t, true), rd = run_length(J, dst_order, t, false);
      t[(size_t)k] = old;
      if (!fits) continue;
      int64_t mn = std::min(rs, rd), sm = rs + rd;
      if (mn > best_min || (mn == best_min && sm > best_sum)) { best = k; best_min = mn; best_sum = sm; best_t = grown; }
    }
    if (best < 0) break;
    const int64_t cur_s = run_length(J, src_order, t, true), cur_d = run_length(J, dst_order, t, false);
    if (tune.micro_per_thread <= 0 && micro_of(t) >= full_wg && std::min(cur_s, cur_d) * es >= enough_run_bytes) break;
    t[(size_t)best] = best_t;
    micro = micro_of(t);
  }
  for (; !ragged;) {
    int best = -1;
    int64_t best_min = -1, best_sum = -1, best_f = 1;
    for (int k = 0; k < nj; ++k) {
      int64_t left = J[(size_t)k].extent / t[(size_t)k];
      if (left <= 1) continue;
      int64_t f = smallest_prime_factor(left);
      if (micro * f > target) continue;
      t[(size_t)k] *= f;
      const bool fits = spans_fit(t);
      int64_t rs = run_length(J, src_order, t, true), rd = run_length(J, dst_order, t, false);
      t[(size_t)k] /= f;
      if (!fits) continue;
      int64_t mn = std::min(rs, rd), sm = rs + rd;
      if (mn > best_min || (mn == best_min && sm > best_sum)) { best = k; best_min = mn; best_sum = sm; best_f = f; }
    }
    if (best < 0) break;
    const int64_t cur_s = run_length(J, src_order, t, true), cur_d = run_length(J, dst_order, t, false);
    int64_t cur_min = std::min(cur_s, cur_d), cur_sum = cur_s + cur_d;
    if (best_min <= cur_min && best_sum <= cur_sum) break;   // growing further no longer lengthens any run
    if (tune.micro_per_thread <= 0 && micro >= full_wg && cur_min * es >= enough_run_bytes) break;   // runs are long enough: keep more tiles
    t[(size_t)best] *= best_f;
    micro *= best_f;
  }
  if (tune.tile.size() == (size_t)nj && !ragged) {   // explicit tile (tuning): must divide the extents and hold whole micro-tiles
    bool valid = true;
    int64_t m2 = 1;
    for (int k = 0; k < nj; ++k) {
      int64_t te = tune.tile[(size_t)k];
      if (te < 1 || J[(size_t)k].extent % te != 0 || ((k == p || k == q) && te % V != 0)) valid = false;
      else m2 *= (k == p || k == q) ? te / V : te;
    }
    if (valid && m2 <= (int64_t)max_per_lane * kBlock) { t = tune.tile; micro = m2; }
  }
  // no run can be lengthened any more: still fill the workgroup, smallest destination strides first
  for (int k = 0; k < nj && tune.tile.size() != (size_t)nj && !ragged; ++k)
    for (;;) {
      int64_t left = J[(size_t)k].extent / t[(size_t)k];
      int64_t f = left > 1 ? smallest_prime_factor(left) : 0;
      if (f == 0 || micro * f > (tune.micro_per_thread > 0 ? target : std::min<int64_t>(target, full_wg))) break;
      t[(size_t)k] *= f;
      if (!spans_fit(t)) { t[(size_t)k] /= f; break; }
      micro *= f;
    }
  // tiling = zipped_divide of both joint layouts by the tile extents (Sec. 3.5.2): mode 0 is
  // the tile, mode 1 the grid of tiles; a workgroup slices mode 1 with its tile id.
  Modes js, jd, tl;
  for (int k = 0; k < nj; ++k) {
    js.push_back({J[(size_t)k].extent, J[(size_t)k].a});
    jd.push_back({J[(size_t)k].extent, J[(size_t)k].b});
    tl.push_back({t[(size_t)k], 1});
  }
  Layout zs, zd;
  Layout tiler = nj == 1 ? Layout::tuple({Layout::flat(tl)}) : Layout::flat(tl);
  Layout jsl = nj == 1 ? Layout::tuple({Layout::flat(js)}) : Layout::flat(js);
  Layout jdl = nj == 1 ? Layout::tuple({Layout::flat(jd)}) : Layout::flat(jd);
  bool ok = true;
  Layout ts, td, rs_, rd_;
  std::vector<int> ragged_modes;
  for (int k = 0; k < nj; ++k)
    if (J[(size_t)k].extent % t[(size_t)k] != 0) ragged_modes.push_back(k);
  if (ragged_modes.empty()) {
    ok = zipped_divide(jsl, tiler, &zs) == LC_OK && zipped_divide(jdl, tiler, &zd) == LC_OK;
    if (ok) {
      ts = zs.mode(0); td = zd.mode(0); rs_ = zs.mode(1); rd_ = zd.mode(1);
      ok = ts.leaves.size() == (size_t)nj && td.leaves.size() == (size_t)nj && rs_.leaves.size() == rd_.leaves.size();
    }
  } else {
    // the tiler does not divide the shape, so the divide is not admissible (Sec. 3.3.1); the tile and
    // the grid are written down directly: tile mode k = t_k : stride_k, grid mode k = ceil(e_k / t_k) : t_k stride_k
    Modes tsm, tdm, rsm, rdm;
    for (int k = 0; k < nj; ++k) {
      const int64_t e = J[(size_t)k].extent, tk = t[(size_t)k], cnt = (e + tk - 1) / tk;
      tsm.push_back({tk, J[(size_t)k].a}); tdm.push_back({tk, J[(size_t)k].b});
      rsm.push_back({cnt, tk * J[(size_t)k].a}); rdm.push_back({cnt, tk * J[(size_t)k].b});
    }
    ts = Layout::flat(tsm); td = Layout::flat(tdm); rs_ = Layout::flat(rsm); rd_ = Layout::flat(rdm);
    ok = ragged && ragged_modes.size() <= 2;
    for (int k : ragged_modes)   // whole vectors only: the extent along p and q is a multiple of V by the choice of V
      if ((k == p || k == q) && J[(size_t)k].extent % V != 0) ok = false;
  }
  TransposeParams& P = plan->transpose;
  std::memset(&P, 0, sizeof(P));
  int64_t max_in_tile = 0;
  if (ok) {
    // micro modes: the tile box with V taken out of p and q
    struct MM { int64_t ext, sa, sb; bool is_p, is_q; uint32_t cw; };
    std::vector<MM> mm;
    auto coord_weight = [&](int joint_mode, int64_t step) -> uint32_t {   // packed coordinate step along the ragged modes
      for (size_t j = 0; j < ragged_modes.size(); ++j)
        if (ragged_modes[j] == joint_mode) return (uint32_t)step << (16 * j);
      return 0u;
    };
    for (int k = 0; k < nj; ++k) {
      int64_t te = ts.leaves[(size_t)k].extent, ta = ts.leaves[(size_t)k].stride, tb = td.leaves[(size_t)k].stride;
      if (te != t[(size_t)k] || td.leaves[(size_t)k].extent != te) { ok = false; break; }
      max_in_tile = std::max(max_in_tile, std::max((te - 1) * ta, (te - 1) * tb));
      int64_t ext = (k == p || k == q) ? te / V : te;
      int64_t scale = (k == p || k == q) ? V : 1;
      if (ext > 1) mm.push_back({ext, ta * scale, tb * scale, k == p, k == q, coord_weight(k, scale)});
    }
    int64_t span_s = 0, span_d = 0;
    for (int k = 0; k < nj; ++k) { span_s += (t[(size_t)k] - 1) * std::abs(J[(size_t)k].a); span_d += (t[(size_t)k] - 1) * J[(size_t)k].b; }
    if (span_s >= (1ll << 30) || span_d >= (1ll << 30) || mm.size() >= (size_t)kMaxModes) ok = false;
    if (ok) {
      // destination order of the tile's vectors: the micro modes and the position ip along p
      // inside a micro-tile (extent V, destination stride b_p), by destination stride, q first
      mm.push_back({V, 0, J[(size_t)p].b, false, false, coord_weight(p, 1)});
      const int pv = (int)mm.size() - 1;
      std::vector<int> so, dord;
      for (int k = 0; k < (int)mm.size(); ++k) { if (k != pv) so.push_back(k); dord.push_back(k); }
      std::stable_sort(so.begin(), so.end(), [&](int x, int y) {
        if (mm[(size_t)x].is_p != mm[(size_t)y].is_p) return mm[(size_t)x].is_p;
        return mm[(size_t)x].sa < mm[(size_t)y].sa; });
      std::stable_sort(dord.begin(), dord.end(), [&](int x, int y) {
        if (mm[(size_t)x].is_q != mm[(size_t)y].is_q) return mm[(size_t)x].is_q;
        return mm[(size_t)x].sb < mm[(size_t)y].sb; });
      std::vector<uint32_t> gpos(mm.size(), 0);
      uint32_t run = 1;
      for (size_t j = 0; j < dord.size(); ++j) {
        const MM& m = mm[(size_t)dord[j]];
        P.ext_d[j] = make_fastdiv((uint32_t)m.ext);
        P.sb_d[j] = (int32_t)m.sb;
        P.cw_d[j] = m.cw;
        gpos[(size_t)dord[j]] = run;
        run *= (uint32_t)m.ext;
      }
      P.n_dst_modes = (int32_t)dord.size();
      P.gpos_pv = gpos[(size_t)pv];
      for (size_t j = 0; j < so.size(); ++j) {
        const MM& m = mm[(size_t)so[j]];
        P.ext_s[j] = make_fastdiv((uint32_t)m.ext);
        P.sa_s[j] = (int32_t)m.sa;
        P.gpos_s[j] = gpos[(size_t)so[j]];
        P.cw_s[j] = m.cw;
      }
      P.n_micro_modes = (int32_t)so.size();
      // lane / trip split of the two decodes (see TransposeParams)
      P.src_split = P.dst_split = 0;
      {
        // number of leading modes the lane index reaches into, when lane + i * kBlock decodes without
        // a carry between the two terms: the modes below the last are covered by the lane alone, and
        // in the last one the lane's digit stays below a divisor c of the extent while i moves it in
        // steps of c.  0 when extents and kBlock do not nest that way.
        auto split_of = [](const FastDiv* ext, int n_modes) -> int {
          uint64_t prod = 1;
          for (int k = 0; k < n_modes; ++k) {
            const uint64_t c = (uint64_t)kBlock / prod;
            if (c == 1) return k;
            if (ext[k].div % c == 0) return k + 1;
            if (c % ext[k].div != 0) return 0;
            prod *= ext[k].div;
          }
          return 0;
        };
        P.src_split = split_of(P.ext_s, P.n_micro_modes);
        P.dst_split = split_of(P.ext_d, P.n_dst_modes);
        // the trips' parts: decode i * kBlock in full (its lane digits are zero)
        for (int i = 0; i < kMaxMicroPerLane; ++i) {
          P.src_trip_off[i] = 0;
          P.src_trip_g[i] = 0;
          if (P.src_split > 0 && (uint64_t)i * kBlock < run / (uint32_t)V)
            micro_from_src_order(P, (uint32_t)i * kBlock, &P.src_trip_off[i], &P.src_trip_g[i]);
        }
        for (int i = 0; i < kMaxPicksPerLane; ++i)
          P.dst_trip_off[i] = (P.dst_split > 0 && (uint64_t)i * kBlock < run) ? vector_dst_offset(P, (uint32_t)i * kBlock) : 0;
      }
      P.n_vec = run;
      P.n_micro = run / (uint32_t)V;
      P.a_q = (int32_t)J[(size_t)q].a;
      if (std::abs(J[(size_t)q].a) * (V - 1) >= (1ll << 30) || J[(size_t)p].b * (V - 1) >= (1ll << 30)) ok = false;
    }
  }
  if (ok) {
    // rest modes = grid of tiles
    struct RM { int64_t ext, a, b; int joint; };
    std::vector<RM> rest;
    if (!ragged_modes.empty() && rs_.leaves.size() != (size_t)nj) ok = false;
    for (size_t k = 0; k < rs_.leaves.size() && ok; ++k) {
      if (rs_.leaves[k].extent != rd_.leaves[k].extent) { ok = false; break; }
      if (rs_.leaves[k].extent > 1) rest.push_back({rs_.leaves[k].extent, rs_.leaves[k].stride, rd_.leaves[k].stride, (int)k});
    }
    // Tile ids run fastest along the smallest SOURCE stride: resident workgroups then read one
    // contiguous region together (measured 1-3 % better than destination order; writes are combined
    // by the caches anyway).
    if (tune.rest_order != 0)
      std::stable_sort(rest.begin(), rest.end(), [](const RM& x, const RM& y) { return x.a < y.a; });
    int64_t tiles = 1;
    for (const RM& r : rest) tiles *= r.ext;
    if (rest.size() > (size_t)kMaxModes || tiles >= (1ll << 31)) ok = false;
    if (ragged_modes.empty() ? tiles * (int64_t)P.n_micro * V * V != n : tiles * (int64_t)P.n_micro * V * V < n) ok = false;
    if (ok) {
      P.n_ragged = (int32_t)ragged_modes.size();
      for (size_t j = 0; j < ragged_modes.size(); ++j) {
        P.rag_extent[j] = (uint32_t)J[(size_t)ragged_modes[j]].extent;
        P.rag_tile[j] = (uint32_t)t[(size_t)ragged_modes[j]];
        P.rag_rest[j] = -1;
        for (size_t k = 0; k < rest.size(); ++k)
          if (rest[k].joint == ragged_modes[j]) P.rag_rest[j] = (int32_t)k;
      }
      P.n_rest = (int32_t)rest.size();
      for (size_t k = 0; k < rest.size(); ++k) {
        P.rdiv[k] = make_fastdiv((uint32_t)rest[k].ext);
        P.ra[k] = rest[k].a;
        P.rb[k] = rest[k].b;
      }
      P.n_tiles = (uint32_t)tiles;
      P.blocked = tune.blocked > 0 ? 1u : 0u;
    }
  }
  if (ok) {
    // a10: where the tile's vectors lie in LDS.  Vector g (destination order) goes to slot g ^ swz(g): an XOR layout over
    // the bits of g (Sec. 2.3.2).  Picks read consecutive g and are conflict-free for any swz that only folds higher bits
    // into the low ones.  Parks: a write pass is nb = log2(128 / slot bytes) consecutive lanes (128 bytes of banks), so the
    // slots' low nb bits have to take every value over the lanes' low nb bits.  With power-of-two extents the park
    // layout lane -> g moves lane bit i to one bit pi(i) of g: a bit that lands below nb already selects a bank bit; every
    // other one is folded onto a bank bit that is still free, i.e. bit pi(i) of g gets the stride f_(2^pi(i) + 2^k) in
    // place of f_(2^pi(i)).  Folds with the same distance pi(i) - k make one shift-and-mask term; the kernels evaluate two.
    // Other shapes (or more terms) fall back to a search over single shifts against the bank model, which in every case
    // has the last word: the derived layout is kept only if the model finds no conflict.
    const int slot_bytes = V * es;
    int nb = 0;
    while ((128 >> (nb + 1)) >= std::max(4, std::min(16, slot_bytes))) ++nb;   // lanes per write pass = 2^nb
    P.swz_shift = P.swz_mask = P.swz_shift2 = P.swz_mask2 = 0;
    bool derived = false;
    if (tune.swizzle_shift == -2 && P.n_micro >= (1u << nb)) {
      uint32_t free_bits = (1u << nb) - 1u;
      int fold_from[8], n_fold = 0;
      bool linear = true;
      for (int i = 0; i < nb && linear; ++i) {
        int32_t so;
        uint32_t g = 0, g_zero = 0;
        micro_from_src_order(P, 1u << i, &so, &g);
        micro_from_src_order(P, 0, &so, &g_zero);
        g -= g_zero;
        if (g == 0 || (g & (g - 1)) != 0) { linear = false; break; }   // the lane bit does not move exactly one bit of g
        int b = 0;
        while ((1u << b) != g) ++b;
        if (b < nb) free_bits &= ~(1u << b);
        else fold_from[n_fold++] = b;
      }
      // and the lanes of a pass really are those bits' span: lane = sum of its bits without carries (power-of-two extents)
      for (int i = 0; i < nb && linear; ++i)
        for (int j = i + 1; j < nb && linear; ++j) {
          int32_t so;
          uint32_t gi = 0, gj = 0, gij = 0;
          micro_from_src_order(P, 1u << i, &so, &gi);
          micro_from_src_order(P, 1u << j, &so, &gj);
          micro_from_src_order(P, (1u << i) | (1u << j), &so, &gij);
          if (gij != gi + gj) linear = false;
        }
      if (linear) {
        uint32_t shift_of[2] = {0, 0}, mask_of[2] = {0, 0};
        int terms = 0;
        bool fits = true;
        for (int f = 0; f < n_fold && fits; ++f) {
          int k = 0;
          while (!(free_bits & (1u << k))) ++k;                          // lowest bank bit still free
          free_bits &= ~(1u << k);
          const uint32_t dist = (uint32_t)(fold_from[f] - k);
          int t = 0;
          while (t < terms && shift_of[t] != dist) ++t;
          if (t == terms) { if (terms == 2) { fits = false; break; } shift_of[terms++] = dist; }
          mask_of[t] |= 1u << k;
        }
        if (fits) {
          P.swz_shift = shift_of[0]; P.swz_mask = mask_of[0];
          P.swz_shift2 = shift_of[1]; P.swz_mask2 = mask_of[1];
          derived = transpose_swizzle_cost(P, V, es, 1u << 20, 64) == 0;
          if (!derived) P.swz_shift = P.swz_mask = P.swz_shift2 = P.swz_mask2 = 0;
        }
      }
    }
    if (!derived) {
      int best_shift = -1;
      int best_cost = transpose_swizzle_cost(P, V, es, 4, 64);
      if (tune.swizzle_shift == -2) {
        for (int sh = 3; best_cost > 0 && sh <= 12 && (P.n_vec >> sh) > 0; ++sh) {
          P.swz_shift = (uint32_t)sh; P.swz_mask = 15;
          int c = transpose_swizzle_cost(P, V, es, 4, 64);
          if (c < best_cost) { best_cost = c; best_shift = sh; }
        }
      } else if (tune.swizzle_shift >= 3) {
        best_shift = tune.swizzle_shift;
      }
      if (best_shift >= 3) { P.swz_shift = (uint32_t)best_shift; P.swz_mask = 15; }
      else { P.swz_shift = 0; P.swz_mask = 0; }
    }
    plan->swizzle_derived = derived;
    plan->cls = KernelClass::Transpose;
    plan->V = V;
    plan->width_bytes = V * es;
    plan->micro_per_thread = (int)((P.n_micro + kBlock - 1) / kBlock);
    if (plan->micro_per_thread == 3) plan->micro_per_thread = 4;
    if (plan->micro_per_thread > 4) plan->micro_per_thread = 8;
    plan->tile_elem_bytes = es;
    plan->tile_extent = t;
    plan->p_mode = p;
    plan->q_mode = q;
    plan->lds_bytes = ((P.n_vec + 15u) & ~15u) * (unsigned)(V * es);
    plan->src_run_bytes = run_length(J, src_order, t, true) * es;
    plan->dst_run_bytes = run_length(J, dst_order, t, false) * es;
    // nontemporal stores only when every store instruction covers whole 128-byte lines
    if (tune.nontemporal < 0 && plan->dst_run_bytes % 128 == 0) plan->nontemporal |= 2;
    // Measured on MI355X: HBM efficiency is best with ONE resident workgroup per CU (its next tile's
    // loads overlap its current tile's stores); short grids need more workgroups to fill the chip.
    int fit = (int)(160 * 1024 / std::max(1u, plan->lds_bytes));
    int want = P.n_tiles >= 16384 ? 1 : (P.n_tiles >= 4096 ? 2 : (P.n_tiles >= 2048 ? 3 : 4));
    // the ragged / element-wise kernel has no software pipeline: resident workgroups overlap each other instead
    if (P.n_ragged > 0 || (V == 1 && es != 16)) want = 8;
    plan->wgs_per_cu = tune.wgs_per_cu > 0 ? tune.wgs_per_cu : std::max(1, std::min(std::min(8, fit), want));
    // Long grids of large tiles: workgroups drift apart over hundreds of tiles, and asking a device-side queue for the
    // next tiles (one request ahead) evens that out.  Measured on MI355X: one request per 64 KiB of tile data is best
    // (64 KiB tiles one at a time: 71 -> 79 % of the HBM peak; 32 KiB tiles two at a time: 73 -> 81 %, one at a time 65 %:
    // too many requests for one counter); with few tiles per workgroup the fixed order is faster (2048 tiles: 69 -> 45 %).
    // 16 bytes of LDS behind the tile carry the answer to the other lanes.  tile_queue = tiles per request, 0 = fixed order.
    const bool queue_fits = (uint64_t)(plan->lds_bytes + 16u) * (unsigned)plan->wgs_per_cu <= 160u * 1024u && !P.blocked &&
                            P.n_ragged == 0 && !(V == 1 && es != 16);   // the kernel without predicates only
    const bool queue_pays = plan->lds_bytes >= 32u * 1024u && P.n_tiles >= 4096u;
    const int per_request = (int)std::max(1u, 65536u / std::max(1u, plan->lds_bytes));
    plan->tile_queue = queue_fits ? (tune.tile_queue >= 0 ? tune.tile_queue : (queue_pays ? per_request : 0)) : 0;
    plan->queue_static_rounds = tune.queue_rounds >= 1 ? tune.queue_rounds : 1;
    plan->queue_counters = tune.queue_counters >= 1 ? tune.queue_counters : 1;
    plan->leftover_lead = tune.leftover_lead >= 0 ? tune.leftover_lead : 0;
    plan->src_align = (unsigned)(V * es);
    plan->dst_align = (unsigned)(V * es);
    if (tune.early_loads != 0) fill_transpose_head(P, plan->micro_per_thread, &plan->head);
    return true;
  }
  return false;
}

// a3: refine both shapes to one shape F by composing each layout with the identity layout of F (Sec. 3.3.1); then every
// mode of F has one stride on each side.  False when the shapes have no common refinement or a composition is not admissible.
static bool joint_modes(const Modes& S, const Modes& D, std::vector<JointMode>* J) {
  std::vector<int64_t> F;
  if (!common_refinement(S, D, &F)) return false;
  Modes ident;
  int64_t run = 1;
  for (int64_t e : F) { ident.push_back({e, run}); run *= e; }
  // Composition is stated for strides in N; a mode of negative stride refines like its mirror image (the same extents,
  // every stride of the refinement with the mode's sign), so the magnitudes are composed and the signs put back.
  auto refine = [&](const Modes& M, std::vector<int64_t>* strides) {
    Modes mag = M;
    for (Mode& m : mag) m.stride = m.stride < 0 ? -m.stride : m.stride;
    Layout R;
    if (composition(Layout::flat(mag), Layout::flat(ident), &R) != LC_OK || R.leaves.size() != F.size()) return false;
    size_t parent = 0;
    int64_t left = M[0].extent;
    for (size_t k = 0; k < F.size(); ++k) {
      while (left == 1 && parent + 1 < M.size()) left = M[++parent].extent;
      strides->push_back(M[parent].stride < 0 ? -R.leaves[k].stride : R.leaves[k].stride);
      left /= F[k];
    }
    return true;
  };
  std::vector<int64_t> sa, sb;
  if (!refine(S, &sa) || !refine(D, &sb)) return false;
  J->clear();
  for (size_t k = 0; k < F.size(); ++k)
    if (F[k] > 1) J->push_back({F[k], sa[k], sb[k]});
  return true;
}

static Modes magnitudes(const Modes& M) {
  Modes out = M;
  for (Mode& m : out) m.stride = m.stride < 0 ? -m.stride : m.stride;
  return out;
}
static bool any_negative(const Modes& M) {
  for (const Mode& m : M) if (m.stride < 0) return true;
  return false;
}

lc_status_t make_plan(const Layout& src, const Layout& dst, int es, unsigned src_align, unsigned dst_align,
                      const Tuning& tune, lc_plan* plan) {
  if (src.size() != dst.size()) return LC_ERR_SIZE_MISMATCH;             // @pre size(src) == size(dst)
  if (es != 1 && es != 2 && es != 4 && es != 8 && es != 16) return LC_ERR_UNSUPPORTED_DTYPE;
  if (src_align == 0 || dst_align == 0 || (src_align & (src_align - 1)) || (dst_align & (dst_align - 1)))
    return LC_ERR_INVALID_ARG;
  const int64_t n = dst.size();
  plan->elem_bytes = es;
  plan->n_elems = n;
  plan->src_align = std::min(src_align, 256u);
  plan->dst_align = std::min(dst_align, 256u);
  plan->nontemporal = tune.nontemporal >= 0 ? (tune.nontemporal & 3) : 1;   // stores: decided per class below
  plan->grid_override = tune.grid > 0 ? tune.grid : 0;
  plan->early_loads = tune.early_loads != 0;

  // a2: both layouts as functions of the integral coordinate (Sec. 3.2)
  Modes S = coalesce_modes(src.leaves), D = coalesce_modes(dst.leaves);
  plan->distinct_reads = 1;
  for (const Mode& m : S)
    if (m.stride != 0) plan->distinct_reads *= m.extent;
  // a1: the destination must be injective, otherwise the result would depend on the iteration order -- except where
  // the order of Sec. 2.6.1's loop (i ascending) decides it without a race: of the coordinates that differ only in
  // destination modes of stride 0, the one with those modes at their last position is written last.  The copy is then
  // the copy of that slice (Sec. 2.5.1): the modes fold into an offset of the source and leave both layouts.
  // (mirroring a mode, c -> extent - 1 - c, turns a negative stride into its magnitude and shifts every offset by the same
  // constant: injectivity is that of the magnitudes)
  if (n > 1 && !layout_is_injective(coalesce_modes(magnitudes(D)), n)) {
    std::vector<JointMode> J0;
    Modes S2, D2;
    int64_t offset = 0, n2 = 1;
    int dropped = 0;
    if (joint_modes(S, D, &J0)) {
      for (const JointMode& m : J0) {
        if (m.b == 0) {
          offset += (m.extent - 1) * m.a;
          ++dropped;
        } else {
          S2.push_back({m.extent, m.a});
          D2.push_back({m.extent, m.b});
          n2 *= m.extent;
        }
      }
    }
    // any other overlap (or a destination too large to enumerate whose strides do not nest): decided per offset on the device
    if (dropped == 0) return plan_last_writer(S, D, n, plan, "destination offsets repeat (or could not be shown distinct)");
    if (S2.empty()) {
      S2.push_back({1, 0});
      D2.push_back({1, 0});
    }
    unsigned shifted_align = plan->src_align;
    while (shifted_align > 1 && (offset * es) % shifted_align != 0) shifted_align /= 2;
    lc_status_t st = make_plan(Layout::flat(S2), Layout::flat(D2), es, shifted_align, dst_align, tune, plan);   // may itself be last-writer
    if (st != LC_OK) return st;
    plan->src_offset_elems += offset;
    plan->overwritten_modes += dropped;
    plan->distinct_reads = 1;
    for (const Mode& m : S)
      if (m.stride != 0) plan->distinct_reads *= m.extent;
    return LC_OK;
  }

  // Negative destination strides: COPY may visit its coordinates in any order as long as both sides take the same one
  // (Sec. 3.4.2), so every joint mode whose destination stride is negative is walked backwards, c -> extent - 1 - c.  Both
  // of its strides change sign and the mode's last element becomes its first: (extent - 1) * stride goes into each
  // pointer.  What is left has destination strides >= 0 and is planned as usual; source strides that are still negative
  // are true reversals of source against destination and stay (the kernels' index arithmetic is signed).
  if (any_negative(D)) {
    std::vector<JointMode> J0;
    if (!joint_modes(S, D, &J0)) return plan_generic(S, D, n, plan, "shapes have no common refinement");   // signed strides as they are
    Modes S2, D2;
    int64_t src_shift = 0, dst_shift = 0;
    for (const JointMode& m : J0) {
      if (m.b < 0) {
        src_shift += (m.extent - 1) * m.a;
        dst_shift += (m.extent - 1) * m.b;
        S2.push_back({m.extent, -m.a});
        D2.push_back({m.extent, -m.b});
      } else {
        S2.push_back({m.extent, m.a});
        D2.push_back({m.extent, m.b});
      }
    }
    if (S2.empty()) { S2.push_back({1, 0}); D2.push_back({1, 0}); }
    auto shifted = [&](unsigned align, int64_t shift) {
      while (align > 1 && (shift * es) % (int64_t)align != 0) align /= 2;
      return align;
    };
    const int64_t reads = plan->distinct_reads;
    lc_status_t st = make_plan(Layout::flat(S2), Layout::flat(D2), es, shifted(plan->src_align, src_shift), shifted(plan->dst_align, dst_shift), tune, plan);
    if (st != LC_OK) return st;
    plan->src_offset_elems += src_shift;
    plan->dst_offset_elems += dst_shift;
    plan->reflected_modes += 1;
    plan->distinct_reads = reads;
    return LC_OK;
  }

  // a5 (the paper's route): K = stride-1 head of src o dst^ (Sec. 3.4.2), reported by describe().  The width the
  // kernels use is derived from the joint modes below and clamped by element width and alignment; when both exist
  // it never exceeds K (asserted where the direct class picks its vector).
  int64_t K = 1;
  const bool K_known = !any_negative(S) && max_common_vector(src, dst, &K) == LC_OK;
  if (!K_known) K = 1;
  plan->common_vector = K;

  // a3: refine both shapes to one shape F by composing each layout with the identity layout of F
  // (Sec. 3.3.1); then every mode of F has one stride on each side.
  std::vector<JointMode> J;
  {
    std::vector<int64_t> F;
    if (!common_refinement(S, D, &F)) return plan_generic(S, D, n, plan, "shapes have no common refinement");
    if (!joint_modes(S, D, &J)) return plan_generic(S, D, n, plan, "refinement by composition was not admissible");
  }
  if (J.empty()) J.push_back({1, 0, 0});

  // a4: the same permutation on both sides leaves COPY unchanged (Sec. 3.4.2): order by destination
  // stride, then merge neighbours that continue each other on both sides.
  std::stable_sort(J.begin(), J.end(), [](const JointMode& x, const JointMode& y) { return x.b != y.b ? x.b < y.b : x.a < y.a; });
  {
    std::vector<JointMode> merged;
    for (const JointMode& m : J) {
      if (!merged.empty() && m.a == merged.back().extent * merged.back().a && m.b == merged.back().extent * merged.back().b)
        merged.back().extent *= m.extent;
      else
        merged.push_back(m);
    }
    J = merged;
  }
  plan->joint = J;
  if (J.size() > (size_t)kMaxModes) return plan_generic(S, D, n, plan, "more joint modes than the tiled kernels index");

  const int nj = (int)J.size();
  int q = -1, p = -1;
  for (int k = 0; k < nj; ++k) {
    if (q < 0 && J[(size_t)k].b == 1) q = k;
    if (p < 0 && J[(size_t)k].a == 1) p = k;
  }
  int cap = 16 / es;
  if (tune.max_vec_bytes > 0) cap = std::max(1, std::min(cap, tune.max_vec_bytes / es));
  cap = std::max(1, std::min<int>(cap, (int)std::min(plan->src_align, plan->dst_align) / es));

  // ---- Transpose class: p and q exist and differ -------------------------------------------
  bool want_transpose = (p >= 0 && q >= 0 && p != q) && tune.force_class != 0 && tune.force_class != 1;
  if (want_transpose) {
    std::vector<int64_t> need = {J[(size_t)p].extent, J[(size_t)q].extent};
    for (int k = 0; k < nj; ++k) {
      if (k != p) need.push_back(J[(size_t)k].a);
      if (k != q) need.push_back(J[(size_t)k].b);
    }
    int V = common_pow2(cap, need);
    while (V >= 2 && !transpose_instantiated(es, V)) V /= 2;
    if (V >= 2) {
      const bool exact = plan_tiled(J, es, V, p, q, n, tune, plan);
      // Whole tiles need extents with small factors.  When they leave runs shorter than a cache line
      // (prime-ish extents) the ragged tiling is tried too and taken if its shorter run is at least twice
      // as long (its kernel is not pipelined: 4000 x 4000 fp32 runs at 63 % with whole 160 x 32 tiles and
      // at 57 % with ragged 128 x 64 tiles, but 8000 x 8008 bf16 at 34 % against 46 %).
      if (exact && (std::min(plan->src_run_bytes, plan->dst_run_bytes) >= 128 || tune.tile.size() == (size_t)nj)) return LC_OK;
      lc_plan rag = *plan;
      rag.cls = KernelClass::Generic;
      if (plan_tiled(J, es, V, p, q, n, tune, &rag, true) && rag.transpose.n_ragged > 0 &&
          (!exact || std::min(rag.src_run_bytes, rag.dst_run_bytes) >= 2 * std::min(plan->src_run_bytes, plan->dst_run_bytes))) {
        *plan = rag;
        return LC_OK;
      }
      if (exact) return LC_OK;
      plan->note = "tile did not fit the transpose kernel's index ranges";
    } else {
      // No vector on one side (odd strides or extents): single elements through the same tiles (V = 1).
      // In destination order a lane would read one element per source line; a tile reads and writes runs.
      lc_plan rag = *plan;
      if (ragged_instantiated(es, 1) && plan_tiled(J, es, 1, p, q, n, tune, &rag, true) &&
          std::min(rag.src_run_bytes, rag.dst_run_bytes) >= 8 * es) {
        *plan = rag;
        return LC_OK;
      }
      plan->note = "no common vector on both sides for a transposing tile";
    }
  }
  if (tune.force_class == 0) return plan_generic(S, D, n, plan, "forced");

  // ---- Direct class: lanes follow the destination order --------------------------------------
  int VEC = 1;
  if (q >= 0 && J[(size_t)q].a == 1) {
    std::vector<int64_t> need = {J[(size_t)q].extent};
    for (int k = 0; k < nj; ++k)
      if (k != q) { need.push_back(J[(size_t)k].a); need.push_back(J[(size_t)k].b); }
    VEC = common_pow2(cap, need);
    // the two routes to the vector agree: a run that both sides keep contiguous is a prefix of the algebraic K
    if (K_known && VEC > K) VEC = common_pow2((int)std::min<int64_t>(cap, K), need);
  }
  // Gather with a small source stride S along the destination-contiguous mode (S * es < 32 bytes: every 16-byte word of
  // the source span holds a wanted element): whole 16-byte words on both sides.  Vector o of the destination takes its
  // 16 / es elements from the S consecutive words S * o .. S * o + S - 1, so in units of words the mode has source stride S
  // and destination stride 1, and every other stride has to be a whole number of words on both sides.
  // Measured on MI355X (stride 3, 2^26 fp32): 59 % of the HBM peak against 82 % element by element -- a lane's three words
  // lie 48 bytes from its neighbour's, so each load instruction touches every cache line of the span and the span crosses
  // the vector cache three times, while element-wise lanes (one element each, 12 bytes apart) touch each line once per
  // side and already run at the memory system's pace.  The path is therefore taken on request only (LC_TUNE_GATHER=1).
  plan->gather_stride = 0;
  if (q == 0 && VEC == 1 && tune.gather > 0 && (es == 2 || es == 4 || es == 8) && cap == 16 / es) {
    const int64_t S = J[0].a, VE = 16 / es;
    bool fits = S >= 2 && S <= 7 && S * es < 32 && J[0].extent % VE == 0 && J[0].extent / VE >= 2;
    for (int k = 1; k < nj && fits; ++k)   // (a source mode of stride 0 would be looped inside the lane: the direct kernel's job)
      if (J[(size_t)k].a == 0 || J[(size_t)k].a % VE != 0 || J[(size_t)k].b % VE != 0) fits = false;
    if (fits) {
      VEC = (int)VE;
      plan->gather_stride = (int)S;
    }
  }

  // ---- Transpose class on 16-byte words ---------------------------------------------------------
  // The common vector keeps whole 16-byte words together on both sides (p = q), but it is short: in
  // destination order the source would be read in pieces of K elements.  With the word as the
  // element the copy is a permutation of words, and a tile through LDS (V = 1: nothing to transpose
  // inside a word) reads and writes runs of many words.  Measured on MI355X (2^25..2^27 bf16 elements):
  // 128-byte pieces 59 % of the HBM peak in destination order, 71 % through tiles; 256-byte pieces
  // run at 72-73 % either way and stay with the direct class.
  {
    const int64_t direct_run_bytes = q >= 0 ? J[(size_t)q].extent * es : es;
    bool stage = VEC * es == 16 && q >= 0 && p == q && nj >= 3 && direct_run_bytes < 256 && tune.force_class != 1;
    for (int k = 0; k < nj && stage; ++k)
      if (J[(size_t)k].a == 0) stage = false;   // broadcasts are looped inside a lane by the direct class
    if (stage) {
      std::vector<JointMode> W;
      for (int k = 0; k < nj; ++k) {
        JointMode m = J[(size_t)k];
        if (k == q) m.extent /= VEC; else { m.a /= VEC; m.b /= VEC; }
        if (m.extent > 1) W.push_back(m);
      }
      int pw = 0, qw = 0;   // modes of the smallest source / destination stride
      for (int k = 1; k < (int)W.size(); ++k) {
        if (W[(size_t)k].a < W[(size_t)pw].a) pw = k;
        if (W[(size_t)k].b < W[(size_t)qw].b) qw = k;
      }
      lc_plan staged = *plan;
      if (W.size() >= 2 && plan_tiled(W, 16, 1, pw, qw, n / VEC, tune, &staged) &&
          (tune.force_class == 2 || (staged.src_run_bytes >= 4 * direct_run_bytes && staged.dst_run_bytes >= 4 * direct_run_bytes &&
                                     staged.transpose.n_tiles >= 256))) {
        *plan = staged;
        return LC_OK;
      }
    }
  }
  DirectParams& P = plan->direct;
  std::memset(&P, 0, sizeof(P));
  // a stride-0 source mode (broadcast) is looped inside the lane: one read, many writes
  int loop_mode = -1;
  for (int k = 0; k < nj; ++k)
    if (J[(size_t)k].a == 0 && J[(size_t)k].extent > 1 && k != q && J[(size_t)k].extent <= 65536 &&
        (loop_mode < 0 || J[(size_t)k].extent > J[(size_t)loop_mode].extent))
      loop_mode = k;
  // Work items are indexed with 31 bits.  A larger copy is cut along its outermost joint mode into
  // equal slices, one launch per slice (a slice is a pointer offset, Sec. 2.5.1).
  std::vector<JointMode> Jd = J;
  {
    int64_t total = 1;
    int outer = -1;
    for (int k = 0; k < nj; ++k) {
      if (k == loop_mode) continue;
      total *= (k == q) ? Jd[(size_t)k].extent / VEC : Jd[(size_t)k].extent;
      outer = k;
    }
    const int64_t limit = tune.max_items > 0 ? tune.max_items : (1ll << 31) - 1;
    if (total > limit && outer >= 0) {
      int64_t ext = (outer == q) ? Jd[(size_t)outer].extent / VEC : Jd[(size_t)outer].extent;
      int64_t need = (total + limit - 1) / limit, cuts = 0;
      for (int64_t c = need; c <= ext && c < need + (1 << 20); ++c)
        if (ext % c == 0) { cuts = c; break; }
      if (cuts == 0) return LC_ERR_TOO_LARGE;
      Jd[(size_t)outer].extent /= cuts;
      plan->n_launches = cuts;
      plan->launch_src_step = Jd[(size_t)outer].extent * Jd[(size_t)outer].a;
      plan->launch_dst_step = Jd[(size_t)outer].extent * Jd[(size_t)outer].b;
    }
  }
  int64_t items = 1;
  int m = 0;
  for (int k = 0; k < nj; ++k) {
    if (k == loop_mode) continue;
    int64_t ext = Jd[(size_t)k].extent, a = Jd[(size_t)k].a, b = Jd[(size_t)k].b;
    if (k == q && VEC > 1) ext /= VEC; else { a /= (k == q ? 1 : VEC); b /= (k == q ? 1 : VEC); }
    P.div[m] = make_fastdiv((uint32_t)ext);
    P.sa[m] = a;
    P.sb[m] = b;
    items *= ext;
    ++m;
  }
  if (m == 0) { P.div[0] = make_fastdiv(1); P.sa[0] = 0; P.sb[0] = 0; m = 1; }
  if (items >= (1ll << 31)) return LC_ERR_TOO_LARGE;
  P.n_modes = m;
  P.n_items = (uint32_t)items;
  P.loop_extent = loop_mode >= 0 ? (uint32_t)J[(size_t)loop_mode].extent : 1u;
  P.loop_sa = loop_mode >= 0 ? J[(size_t)loop_mode].a / VEC : 0;
  P.loop_sb = loop_mode >= 0 ? J[(size_t)loop_mode].b / VEC : 0;
  P.blocked = tune.blocked > 0 ? 1u : 0u;
  plan->cls = KernelClass::Direct;
  plan->width_bytes = VEC * es;
  // about 16 KiB of accesses in flight per CU measured best on MI355X: unroll x workgroups = 64 / width
  const int W = VEC * es;
  int dflt_unroll = W >= 16 ? 2 : (W >= 4 ? 4 : 8), dflt_wgs = W >= 8 ? 3 : 4;   // 3 x 256 CUs: a grid that is not a power of two
  plan->unroll = (tune.unroll == 1 || tune.unroll == 2 || tune.unroll == 4 || tune.unroll == 8) ? tune.unroll : dflt_unroll;
  plan->wgs_per_cu = tune.wgs_per_cu > 0 ? tune.wgs_per_cu : dflt_wgs;
  // Contiguous copies of 2 GiB and more per side: the grid-stride order lets workgroups drift apart, chunks of 32 KiB handed
  // out to the wavefronts on request keep what is in flight together (measured on MI355X, plain copy, fixed order -> chunks:
  // 2 x 4 GiB 72 -> 77 % of the HBM peak, 2 x 2 GiB 72-75 -> 76-77 %; 2 x 1 GiB 72-78 (by where the buffers lie) -> 74-75 %,
  // 2 x 512 MiB 76 -> 70 %, the stride-3 gather of 256 MiB 82 -> 70 %: those stay with the fixed order).  Two workgroups per
  // CU and eight counters measured best.
  {
    const int64_t dst_bytes = items * W * (int64_t)P.loop_extent;
    const bool contiguous = P.n_modes == 1 && P.loop_extent == 1 && std::abs(P.sa[0]) == 1 && std::abs(P.sb[0]) == 1;
    const int kib = tune.direct_queue >= 0 ? tune.direct_queue : (dst_bytes >= (2ll << 30) && contiguous && plan->gather_stride == 0 ? 32 : 0);
    plan->direct_queue_items = kib > 0 ? (int)std::max<int64_t>(64 * plan->unroll, (int64_t)kib * 1024 / W) : 0;
    if (plan->direct_queue_items > 0) {
      if (tune.wgs_per_cu <= 0) plan->wgs_per_cu = 2;
      plan->queue_counters = tune.queue_counters >= 1 ? tune.queue_counters : 8;
    }
  }
  if (tune.nontemporal < 0 && ((int64_t)W * (q >= 0 ? J[(size_t)q].extent / VEC : 1)) % 128 == 0) plan->nontemporal |= 2;
  plan->src_align = (unsigned)(VEC * es);
  plan->dst_align = (unsigned)(VEC * es);
  return LC_OK;
}

std::string describe(const lc_plan& plan) {
  std::string s;
  const char* cls = plan.cls == KernelClass::Generic ? "generic" : plan.cls == KernelClass::Direct ? "direct" :
                    plan.cls == KernelClass::LastWriter ? "last-writer" : "transpose";
  s += std::string("class=") + cls;
  s += " elem_bytes=" + std::to_string(plan.elem_bytes) + " n=" + std::to_string(plan.n_elems);
  s += " K=" + std::to_string(plan.common_vector) + " width_bytes=" + std::to_string(plan.width_bytes);
  if (plan.overwritten_modes > 0)
    s += " overwritten_modes=" + std::to_string(plan.overwritten_modes) + " src_offset=" + std::to_string(plan.src_offset_elems);
  if (plan.reflected_modes > 0)
    s += " reflected=1 src_offset=" + std::to_string(plan.src_offset_elems) + " dst_offset=" + std::to_string(plan.dst_offset_elems);
  s += " joint=[";
  for (size_t k = 0; k < plan.joint.size(); ++k) {
    if (k) s += " ";
    s += "(" + std::to_string(plan.joint[k].extent) + "," + std::to_string(plan.joint[k].a) + "," + std::to_string(plan.joint[k].b) + ")";
  }
  s += "]";
  if (plan.cls == KernelClass::Transpose) {
    s += " V=" + std::to_string(plan.V) + " tile_elem_bytes=" + std::to_string(plan.tile_elem_bytes) + " tile=[";
    for (size_t k = 0; k < plan.tile_extent.size(); ++k) { if (k) s += ","; s += std::to_string(plan.tile_extent[k]); }
    s += "] p=" + std::to_string(plan.p_mode) + " q=" + std::to_string(plan.q_mode);
    s += " micro_tiles=" + std::to_string(plan.transpose.n_micro) + " per_lane=" + std::to_string(plan.micro_per_thread);
    s += " tiles=" + std::to_string(plan.transpose.n_tiles) + " lds_bytes=" + std::to_string(plan.lds_bytes);
    s += " swizzle_shift=" + std::to_string(plan.transpose.swz_mask ? (int)plan.transpose.swz_shift : -1);
    s += std::string(" swizzle=") + (plan.swizzle_derived ? "derived" : plan.transpose.swz_mask ? "searched" : "none");
    {
      // the slot function as a layout with XOR strides over the bits of g (Sec. 2.3.2)
      int bits = 0;
      while ((1u << bits) < plan.transpose.n_vec) ++bits;
      std::string shape, stride;
      const TransposeParams& T = plan.transpose;
      for (int b = 0; b < std::max(bits, 1); ++b) {
        uint32_t d = 1u << b;
        if (b >= (int)T.swz_shift && ((T.swz_mask >> (b - (int)T.swz_shift)) & 1u)) d ^= 1u << (b - (int)T.swz_shift);
        if (b >= (int)T.swz_shift2 && ((T.swz_mask2 >> (b - (int)T.swz_shift2)) & 1u)) d ^= 1u << (b - (int)T.swz_shift2);
        shape += (b ? ",2" : "2");
        stride += (b ? ",f" : "f") + std::to_string(d);
      }
      s += " lds_layout=(" + shape + "):(" + stride + ")";
    }
    s += " modelled_lds_conflicts=" + std::to_string(transpose_swizzle_cost(plan.transpose, plan.V, plan.tile_elem_bytes, 1u << 20, 64));
    s += " lane_split=" + std::to_string(plan.transpose.src_split) + "/" + std::to_string(plan.transpose.dst_split);
    s += " ragged_modes=" + std::to_string(plan.transpose.n_ragged);
    s += " early_loads=" + std::to_string(plan.head.ctl & 1u);
    s += " src_run_bytes=" + std::to_string(plan.src_run_bytes) + " dst_run_bytes=" + std::to_string(plan.dst_run_bytes);
  } else if (plan.cls == KernelClass::Direct) {
    s += " items=" + std::to_string(plan.direct.n_items) + " loop=" + std::to_string(plan.direct.loop_extent);
    s += " launches=" + std::to_string(plan.n_launches);
    s += " unroll=" + std::to_string(plan.unroll);
    if (plan.gather_stride) s += " gather_stride=" + std::to_string(plan.gather_stride);
    if (plan.direct_queue_items) s += " chunk_items=" + std::to_string(plan.direct_queue_items) + " queue_counters=" + std::to_string(plan.queue_counters);
    s += " early_loads=" + std::to_string(!plan.gather_stride && plan.early_loads && plan.direct.n_modes == 1 && plan.direct.loop_extent < (1u << 30) ? 1 : 0);
  }
  if (plan.cls == KernelClass::LastWriter) s += " workspace_bytes=" + std::to_string(plan.workspace_bytes);
  s += " wgs_per_cu=" + std::to_string(plan.wgs_per_cu) + " nt=" + std::to_string(plan.nontemporal);
  if (plan.tile_queue)
    s += " tile_queue=" + std::to_string(plan.tile_queue) + " queue_rounds=" + std::to_string(plan.queue_static_rounds) +
         " queue_counters=" + std::to_string(plan.queue_counters);
  if (plan.leftover_lead) s += " leftover_lead=" + std::to_string(plan.leftover_lead);
  s += " blocked=" + std::to_string(plan.cls == KernelClass::Transpose ? plan.transpose.blocked : plan.cls == KernelClass::Direct ? plan.direct.blocked : 0u);
  if (!plan.note.empty()) s += " note=\"" + plan.note + "\"";
  return s;
}

}  // namespace lc
