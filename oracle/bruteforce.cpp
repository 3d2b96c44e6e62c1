// ORACLE — test infrastructure only.
//
// Brute-force checker: runs the oracle's algebra over a universe of small layouts and checks
// every result against the defining post-conditions the paper states for that operation
// (Sec. 3.2 coalesce, Sec. 3.3 composition, Sec. 3.4.1 right-inverse, Sec. 3.5 complement,
// Sec. 3.5.2 divides, Sec. 3.4.2 vectorisation), by enumerating all coordinates.
// The universe: flat shapes of rank 1..R with extents 1..E; for every ordering of the modes the
// compact strides in that ordering; optionally one mode's stride set to 0, optionally the strides
// above one mode scaled by 2 or 3 (padding); every regrouping of the modes into contiguous groups.
// A second universe takes every stride in 0..Dmax for rank <= 3, extents <= 4.
//
// usage: bruteforce [--rank R] [--extent E] [--pair-rank r] [--pair-extent e] [--random N] [--seed S] [--product-budget C]
//                   [--phases unary,pairs,random] [--pair-slice k/n]   (a long run can be cut into parts whose tallies add up)
// Exit status 0 iff no post-condition failed.
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <numeric>
#include <string>
#include <vector>

#include "layout_oracle.hpp"

using namespace oracle;

namespace {

struct Tally {
  std::atomic<long> cases{0}, ok{0}, fail{0};
  std::mutex mu;
  std::string first_failure;
  void failed(const std::string& what) {
    fail++;
    std::lock_guard<std::mutex> g(mu);
    if (first_failure.empty()) first_failure = what;
  }
};
std::map<std::string, Tally> tallies;
Tally& tally(const char* name) { return tallies[name]; }   // all names are created before threads start

std::vector<int64_t> image_of(const Layout& L, int64_t n) {
  std::vector<int64_t> v((size_t)n);
  for (int64_t i = 0; i < n; ++i) v[(size_t)i] = eval(L, i);
  return v;
}

bool is_injective(const Layout& L) {
  std::vector<int64_t> v = image_of(L, size(L));
  std::sort(v.begin(), v.end());
  return std::adjacent_find(v.begin(), v.end()) == v.end();
}

// ---- regroupings of a flat layout into contiguous groups --------------------------------------
Layout regroup(const std::vector<int64_t>& s, const std::vector<int64_t>& d, unsigned cuts) {
  // bit k of cuts set -> a group boundary between mode k and mode k+1; groups of one mode stay ints
  std::vector<Layout> groups;
  size_t start = 0;
  for (size_t k = 0; k < s.size(); ++k) {
    bool end = (k + 1 == s.size()) || ((cuts >> k) & 1u);
    if (!end) continue;
    std::vector<int64_t> gs(s.begin() + (long)start, s.begin() + (long)k + 1), gd(d.begin() + (long)start, d.begin() + (long)k + 1);
    groups.push_back(make_layout(gs, gd));
    start = k + 1;
  }
  if (groups.size() == 1 && s.size() > 1) return groups[0];   // one group = the flat layout itself
  if (groups.size() == 1) return groups[0];
  return concat(groups);
}

// ---- universe -----------------------------------------------------------------------------------
void flat_universe(int max_rank, int max_extent, std::vector<std::pair<std::vector<int64_t>, std::vector<int64_t>>>* out) {
  for (int r = 1; r <= max_rank; ++r) {
    std::vector<int64_t> s((size_t)r, 1);
    for (;;) {
      std::vector<int> perm((size_t)r);
      std::iota(perm.begin(), perm.end(), 0);
      do {
        // compact strides when the modes are laid out in the order perm[0], perm[1], ...
        for (int zero = -1; zero < r; ++zero)
          for (int padpos = -1; padpos < r; ++padpos)
            for (int pad = (padpos < 0 ? 1 : 2); pad <= (padpos < 0 ? 1 : 3); ++pad) {
              std::vector<int64_t> d((size_t)r);
              int64_t run = 1;
              for (int k = 0; k < r; ++k) {
                int m = perm[(size_t)k];
                d[(size_t)m] = run;
                run *= s[(size_t)m];
                if (k == padpos) run *= pad;
              }
              if (zero >= 0) d[(size_t)zero] = 0;
              out->push_back({s, d});
            }
      } while (std::next_permutation(perm.begin(), perm.end()));
      int k = 0;
      while (k < r && s[(size_t)k] == max_extent) { s[(size_t)k] = 1; ++k; }
      if (k == r) break;
      s[(size_t)k]++;
    }
  }
}

void stride_universe(int max_rank, int max_extent, int max_stride, std::vector<std::pair<std::vector<int64_t>, std::vector<int64_t>>>* out) {
  for (int r = 1; r <= max_rank; ++r) {
    std::vector<int64_t> s((size_t)r, 1);
    for (;;) {
      std::vector<int64_t> d((size_t)r, 0);
      for (;;) {
        out->push_back({s, d});
        int k = 0;
        while (k < r && d[(size_t)k] == max_stride) { d[(size_t)k] = 0; ++k; }
        if (k == r) break;
        d[(size_t)k]++;
      }
      int k = 0;
      while (k < r && s[(size_t)k] == max_extent) { s[(size_t)k] = 1; ++k; }
      if (k == r) break;
      s[(size_t)k]++;
    }
  }
}

// ---- unary checks -----------------------------------------------------------------------------------
void check_unary(const Layout& A) {
  const int64_t n = size(A);
  std::vector<int64_t> img = image_of(A, n);
  const std::string name = to_string(A);

  {  // coalesce, Sec. 3.2: |R| = |A|, depth(R) <= 1, R(i) = A(i)
    Tally& t = tally("coalesce");
    t.cases++;
    Layout R = coalesce(A);
    bool good = size(R) == n && depth(R.shape) <= 1;
    for (int64_t i = 0; good && i < n; ++i) good = eval(R, i) == img[(size_t)i];
    // the reading taken: no extent-1 modes (except 1:0) and no mergeable neighbours; idempotent
    std::vector<int64_t> s = leaves(R.shape), d = leaves(R.stride);
    for (size_t k = 0; good && k < s.size(); ++k) {
      if (s[k] == 1 && !(s.size() == 1 && d[0] == 0)) good = false;
      if (k > 0 && d[k] == s[k - 1] * d[k - 1]) good = false;
    }
    if (good && to_string(coalesce(R)) != to_string(R)) good = false;
    if (good) t.ok++; else t.failed("coalesce " + name + " -> " + to_string(R));
  }
  {  // by-mode coalesce: same rank, every mode coalesced on its own, same integral function
    Tally& t = tally("coalesce_bymode");
    t.cases++;
    Layout R = coalesce_bymode(A);
    bool good = size(R) == n && rank(R.shape) == rank(A.shape) && depth(R.shape) <= 2;
    for (int m = 0; good && !A.shape.is_int && m < rank(A.shape); ++m)
      good = size(mode(R.shape, m)) == size(mode(A.shape, m));
    for (int64_t i = 0; good && i < n; ++i) good = eval(R, i) == img[(size_t)i];
    if (good) t.ok++; else t.failed("coalesce_bymode " + name + " -> " + to_string(R));
  }
  bool inj;
  {
    std::vector<int64_t> sorted = img;
    std::sort(sorted.begin(), sorted.end());
    inj = std::adjacent_find(sorted.begin(), sorted.end()) == sorted.end();
  }
  {  // right inverse, Sec. 3.4.1: injective, L(L^(k)) = k, values are coordinates of L, maximal size
    Tally& t = tally("right_inverse");
    t.cases++;
    Layout R = right_inverse(A);
    int64_t m = size(R);
    bool good = m <= n;
    std::vector<int64_t> vals = image_of(R, m);
    for (int64_t k = 0; good && k < m; ++k) good = vals[(size_t)k] >= 0 && vals[(size_t)k] < n && img[(size_t)vals[(size_t)k]] == k;
    std::vector<int64_t> sorted = vals;
    std::sort(sorted.begin(), sorted.end());
    if (good && std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) good = false;
    if (good) t.ok++; else t.failed("right_inverse " + name + " -> " + to_string(R));
    // size bound: |L^| <= K* = largest K with {0..K-1} inside the image; reached when L is injective
    // and the inverse on {0..K*-1} is itself a layout (counted, not required: see report line)
    std::vector<int64_t> simg = img;
    std::sort(simg.begin(), simg.end());
    simg.erase(std::unique(simg.begin(), simg.end()), simg.end());
    int64_t kstar = 0;
    while (kstar < (int64_t)simg.size() && simg[(size_t)kstar] == kstar) ++kstar;
    Tally& tb = tally("right_inverse_size_bound");
    tb.cases++;
    if (m <= kstar) tb.ok++; else tb.failed("right_inverse larger than contiguous image " + name);
    if (inj) {
      // Counted, not required: for an injective L the bound is reached whenever the inverse on
      // {0..K*-1} is itself a layout; the report line shows how often that is the case.
      Tally& tm = tally("right_inverse_maximal_when_injective");
      tm.cases++;
      if (m == kstar) tm.ok++;
    }
  }
  {  // left inverse, Sec. 3.4.3: L(L+(L(k))) = L(k) for every k (L+ evaluated on its extended domain)
    Tally& t = tally("left_inverse");
    t.cases++;
    Layout Li;
    if (left_inverse(A, &Li) == OK) {
      bool good = depth(Li.shape) <= 1;
      for (int64_t k = 0; good && k < n; ++k) good = eval(A, eval(Li, img[(size_t)k])) == img[(size_t)k];
      // injective L: the canonical form L+(L(k)) = k
      if (good && inj) for (int64_t k = 0; good && k < n; ++k) good = eval(Li, img[(size_t)k]) == k;
      if (good) t.ok++; else t.failed("left_inverse " + name + " -> " + to_string(Li));
    }
  }
  {  // complement, Sec. 3.5: ordered image, disjoint images on the extended domain of L*
    for (int variant = 0; variant < 3; ++variant) {
      int64_t co = cosize(A);
      int64_t M = variant == 0 ? 0 : (variant == 1 ? 2 * co : co + 1);
      Tally& t = tally("complement");
      t.cases++;
      Layout C;
      Status st = complement(A, M, &C);
      // completeness: a layout whose non-trivial modes nest exactly must have a complement
      std::vector<int64_t> s = leaves(A.shape), d = leaves(A.stride);
      std::vector<std::pair<int64_t, int64_t>> md;
      for (size_t k = 0; k < s.size(); ++k) if (s[k] > 1 && d[k] > 0) md.push_back({d[k], s[k]});
      std::sort(md.begin(), md.end());
      bool nested = true;
      int64_t cur = 1;
      for (auto& p : md) { if (p.first % cur != 0 || p.first < cur) nested = false; cur = p.first * p.second; }
      if (st != OK) {
        if (nested) t.failed("complement refused a nested layout " + name); else t.ok++;
        continue;
      }
      int64_t cn = size(C);
      bool good = true;
      for (int64_t a = 1; good && a < cn; ++a) good = eval(C, a - 1) < eval(C, a);           // ordered
      std::vector<int64_t> simg = img;
      std::sort(simg.begin(), simg.end());
      for (int64_t a = 1; good && a < 3 * cn + 3; ++a)                                         // disjoint, extended domain
        good = !std::binary_search(simg.begin(), simg.end(), eval(C, a));
      if (good && nested) {
        // (A, A*) is then a bijection onto [0, |A'| |A*|) where A' drops the stride-0 modes, and reaches the cotarget
        int64_t eff = 1;
        for (auto& p : md) eff *= p.second;
        int64_t target = M == 0 ? co : M;
        std::vector<char> seen((size_t)(eff * cn), 0);
        simg.erase(std::unique(simg.begin(), simg.end()), simg.end());
        good = (int64_t)simg.size() == eff && eff * cn >= target;
        for (int64_t a = 0; good && a < cn; ++a)
          for (int64_t v : simg) {
            int64_t o = v + eval(C, a);
            if (o < 0 || o >= eff * cn || seen[(size_t)o]) { good = false; break; }
            seen[(size_t)o] = 1;
          }
      }
      if (good) t.ok++; else t.failed("complement " + name + " under " + std::to_string(M) + " -> " + to_string(C));
    }
  }
}

// ---- pair checks ------------------------------------------------------------------------------------
// The product checks walk size(A) * size(B) coordinates.  Pairs drawn from a large universe can exceed what is
// affordable: above this many coordinates the defining equation of the logical product is checked on an evenly
// spaced lattice of about that many coordinates (both ends included) and the tile-disjointness and
// blocked / raked rearrangement checks, which need the whole image, are left to the smaller pairs.  0 = no limit.
int64_t g_product_budget = 0;

void check_pair(const Layout& A, const Layout& B) {
  const std::string name = to_string(A) + " , " + to_string(B);
  {  // composition, Sec. 3.3: B <= R (compatible) and R(c) = A(B(c)) for every coordinate of B
    Tally& t = tally("composition");
    t.cases++;
    Layout R;
    Status st = composition(A, B, &R);
    if (st == OK) {
      bool good = compatible(B.shape, R.shape);
      for (int64_t c = 0; good && c < size(B); ++c) good = eval(R, c) == eval(A, eval(B, c));
      if (good) t.ok++; else t.failed("composition " + name + " -> " + to_string(R));
    } else {
      // completeness where the paper guarantees it: rank-1 A composes with anything (Sec. 3.3.3)
      // (a trailing extent-1 mode still acts on the extended domain, so it disqualifies A here)
      Layout Ac = coalesce(A);
      std::vector<int64_t> as = leaves(A.shape);
      if (Ac.shape.is_int && (as.size() == 1 || as.back() != 1)) t.failed("composition refused a rank-1 left operand " + name);
      tally("composition_refused").cases++;
    }
  }
  if (size(A) == size(B)) {  // vectorisation, Sec. 3.4.2
    Tally& t = tally("max_common_vector");
    t.cases++;
    int64_t K = 0;
    Status st = max_common_vector_alg(A, B, &K);
    if (st == OK) {
      // meaning of K: for k < K the coordinate B^(k) has offset k in both layouts
      Layout Bi = right_inverse(B);
      bool good = K >= 1 && K <= size(Bi);
      for (int64_t k = 0; good && k < K; ++k) { int64_t c = eval(Bi, k); good = eval(A, c) == k && eval(B, c) == k; }
      // and K is the largest such value
      if (good && K < size(Bi)) { int64_t c = eval(Bi, K); if (eval(A, c) == K) good = false; }
      if (good && is_injective(A) && is_injective(B) && K != max_common_vector_def(A, B)) good = false;
      if (good) t.ok++; else t.failed("max_common_vector " + name + " -> " + std::to_string(K));
    }
  }
  {  // logical product, Sec. 3.5.1: R = (A, A* o B): mode 0 is A, mode 1 is compatible with B,
     // R(a, b) = A(a) + A*(B(b)); tiles are disjoint when A and B are injective and A's modes nest
    Tally& t = tally("logical_product");
    t.cases++;
    Layout R;
    if (logical_product(A, B, &R) == OK) {
      Layout Astar;
      bool good = complement(A, 0, &Astar) == OK && rank(R.shape) == 2 && to_string(sublayout(R, 0)) == to_string(A) &&
                  compatible(B.shape, sublayout(R, 1).shape);
      const int64_t na = size(A), nb = size(B);
      const bool sampled = g_product_budget > 0 && na * nb > g_product_budget;
      int64_t step_a = 1, step_b = 1;
      if (sampled) {
        tally("logical_product_sampled").cases++;
        int64_t side = 1;
        while ((side + 1) * (side + 1) <= g_product_budget) ++side;
        step_a = std::max<int64_t>(1, (na + side - 1) / side);
        step_b = std::max<int64_t>(1, (nb + side - 1) / side);
      }
      for (int64_t b = 0; good && b < nb; b = (b + step_b < nb || b == nb - 1) ? b + step_b : nb - 1)
        for (int64_t a = 0; good && a < na; a = (a + step_a < na || a == na - 1) ? a + step_a : na - 1)
          good = eval(R, a + na * b) == eval(A, a) + eval(Astar, eval(B, b));
      if (good && !sampled && is_injective(A) && is_injective(B)) {
        // the complement is disjoint from A on its whole extended domain, so distinct grid points give disjoint tiles
        std::vector<int64_t> all = image_of(R, na * nb);
        std::sort(all.begin(), all.end());
        // holds when the complement itself is injective over what B asks of it (A's modes nest exactly)
        std::vector<int64_t> as = leaves(A.shape), ad = leaves(A.stride);
        std::vector<std::pair<int64_t, int64_t>> md;
        for (size_t k = 0; k < as.size(); ++k) if (as[k] > 1 && ad[k] > 0) md.push_back({ad[k], as[k]});
        std::sort(md.begin(), md.end());
        bool nested = true;
        int64_t cur = 1;
        for (auto& p : md) { if (p.first % cur != 0) nested = false; cur = p.first * p.second; }
        if (nested && std::adjacent_find(all.begin(), all.end()) != all.end()) good = false;
      }
      if (good) t.ok++; else t.failed("logical_product " + name + " -> " + to_string(R));
    }
    if (rank(A.shape) == rank(B.shape) && !A.shape.is_int && !(g_product_budget > 0 && size(A) * size(B) > g_product_budget)) {
      Tally& tb = tally("blocked_raked_product");
      tb.cases++;
      Layout P, Bp, Rp;
      if (logical_product(A, B, &P) == OK && blocked_product(A, B, &Bp) == OK && raked_product(A, B, &Rp) == OK) {
        // both are rearrangements of the logical product: coordinate ((a_0,b_0),(a_1,b_1),...) resp. ((b_0,a_0),...)
        bool good2 = rank(Bp.shape) == rank(A.shape) && rank(Rp.shape) == rank(A.shape) && size(Bp) == size(P) && size(Rp) == size(P);
        std::vector<int64_t> x = image_of(P, size(P)), y = image_of(Bp, size(Bp)), z = image_of(Rp, size(Rp));
        std::sort(x.begin(), x.end()); std::sort(y.begin(), y.end()); std::sort(z.begin(), z.end());
        if (good2 && (x != y || x != z)) good2 = false;
        for (int i = 0; good2 && i < rank(A.shape); ++i) {
          good2 = to_string(sublayout(sublayout(Bp, i), 0)) == to_string(sublayout(A, i)) &&
                  to_string(sublayout(sublayout(Rp, i), 1)) == to_string(sublayout(A, i));
        }
        if (good2) tb.ok++; else tb.failed("blocked/raked product " + name);
      }
    }
  }
  {  // logical divide, Sec. 3.5.2: R = A o (B, B*_{|A|}); (B, B*) reaches every coordinate of A; mode 0 is A o B
    Tally& t = tally("logical_divide");
    t.cases++;
    Layout R;
    Status st = logical_divide(A, B, &R);
    if (st == OK) {
      Layout Bstar;
      bool good = complement(B, size(A), &Bstar) == OK && rank(R.shape) == 2;
      Layout Bfull = concat({B, Bstar});
      good = good && size(R) == size(Bfull) && size(sublayout(R, 0)) == size(B);
      std::vector<char> hit((size_t)size(A), 0);
      for (int64_t c = 0; good && c < size(R); ++c) {
        int64_t j = eval(Bfull, c);
        good = eval(R, c) == eval(A, j);
        if (j < size(A)) hit[(size_t)j] = 1;
      }
      for (int64_t j = 0; good && j < size(A); ++j) good = hit[(size_t)j] != 0;
      if (good) t.ok++; else t.failed("logical_divide " + name + " -> " + to_string(R));
    }
  }
}

void check_tiler(const Layout& A, const Layout& tiler) {
  if (A.shape.is_int || tiler.shape.is_int || rank(tiler.shape) > rank(A.shape)) return;
  const std::string name = to_string(A) + " , <" + to_string(tiler) + ">";
  Tally& t = tally("zipped_divide");
  t.cases++;
  Layout R;
  if (zipped_divide(A, tiler, &R) != OK) return;
  // Sec. 3.5.2 "Related divides": by-mode logical divide, then like modes zipped:
  // R((t_0,t_1,..),(r_0,r_1,..)) = sum_i (A_i (/) T_i)(t_i, r_i) + sum over untouched modes A_j(r_j)
  bool good = rank(R.shape) == 2;
  std::vector<Layout> D;
  std::vector<int64_t> tsz, rsz;
  for (int i = 0; good && i < rank(A.shape); ++i) {
    if (i < rank(tiler.shape)) {
      Layout Di;
      good = logical_divide(sublayout(A, i), sublayout(tiler, i), &Di) == OK;
      if (!good) break;
      D.push_back(Di);
      tsz.push_back(size(sublayout(Di, 0)));
      rsz.push_back(size(sublayout(Di, 1)));
    } else {
      D.push_back(sublayout(A, i));
      rsz.push_back(size(sublayout(A, i)));
    }
  }
  int64_t T = 1, Rn = 1;
  for (int64_t x : tsz) T *= x;
  for (int64_t x : rsz) Rn *= x;
  good = good && size(sublayout(R, 0)) == T && size(sublayout(R, 1)) == Rn;
  for (int64_t tc = 0; good && tc < T; ++tc)
    for (int64_t rc = 0; good && rc < Rn; ++rc) {
      int64_t expect = 0, tq = tc, rq = rc;
      for (size_t i = 0; i < D.size(); ++i) {
        int64_t ri = rq % rsz[i];
        rq /= rsz[i];
        if (i < tsz.size()) {
          int64_t ti = tq % tsz[i];
          tq /= tsz[i];
          expect += eval(D[i], ti + tsz[i] * ri);
        } else {
          expect += eval(D[i], ri);
        }
      }
      good = eval(R, tc + T * rc) == expect;
    }
  if (good) {  // mode 0 is A composed with the tiler, by mode
    Layout Tl;
    good = composition_bymode(A, tiler, &Tl) == OK;
    std::vector<Layout> tiled;
    for (int i = 0; good && i < rank(tiler.shape); ++i) tiled.push_back(sublayout(Tl, i));
    if (good) {
      Layout tile = tiled.size() == 1 ? tiled[0] : concat(tiled);
      Layout r0 = sublayout(R, 0);
      for (int64_t c = 0; good && c < T; ++c) good = eval(r0, c) == eval(tile, c);
    }
  }
  if (good) t.ok++; else t.failed("zipped_divide " + name + " -> " + to_string(R));
}

uint64_t rng_state = 1;
uint64_t rng() {   // splitmix64
  uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

}  // namespace

int main(int argc, char** argv) {
  int R = 3, E = 4, pr = 2, pe = 4, Dmax = 6;
  long nrandom = 20000;
  uint64_t seed = 2603022980ull;
  bool do_unary = true, do_pairs = true, do_random = true;
  long slice_k = 0, slice_n = 1;   // the pair phase walks the k-th of n slices of the left operands
  for (int i = 1; i + 1 < argc; i += 2) {
    if (!strcmp(argv[i], "--rank")) R = atoi(argv[i + 1]);
    else if (!strcmp(argv[i], "--extent")) E = atoi(argv[i + 1]);
    else if (!strcmp(argv[i], "--pair-rank")) pr = atoi(argv[i + 1]);
    else if (!strcmp(argv[i], "--pair-extent")) pe = atoi(argv[i + 1]);
    else if (!strcmp(argv[i], "--max-stride")) Dmax = atoi(argv[i + 1]);
    else if (!strcmp(argv[i], "--random")) nrandom = atol(argv[i + 1]);
    else if (!strcmp(argv[i], "--seed")) seed = strtoull(argv[i + 1], nullptr, 10);
    else if (!strcmp(argv[i], "--product-budget")) g_product_budget = atoll(argv[i + 1]);
    else if (!strcmp(argv[i], "--phases")) { do_unary = strstr(argv[i + 1], "unary"); do_pairs = strstr(argv[i + 1], "pairs"); do_random = strstr(argv[i + 1], "random"); }
    else if (!strcmp(argv[i], "--pair-slice")) { if (sscanf(argv[i + 1], "%ld/%ld", &slice_k, &slice_n) != 2 || slice_n < 1 || slice_k < 0 || slice_k >= slice_n) { fprintf(stderr, "bad --pair-slice\n"); return 2; } }
    else { fprintf(stderr, "unknown option %s\n", argv[i]); return 2; }
  }
  rng_state = seed;
  for (const char* n : {"coalesce", "coalesce_bymode", "right_inverse", "right_inverse_size_bound",
                        "right_inverse_maximal_when_injective", "complement", "composition", "composition_refused",
                        "max_common_vector", "logical_divide", "zipped_divide", "left_inverse", "logical_product", "logical_product_sampled",
                        "blocked_raked_product"})
    tally(n);

  typedef std::pair<std::vector<int64_t>, std::vector<int64_t>> Flat;
  std::vector<Flat> uni;
  flat_universe(R, E, &uni);
  size_t n_struct = uni.size();
  stride_universe(std::min(R, 3), std::min(E, 4), Dmax, &uni);
  printf("unary universe: %zu structured + %zu small-stride flat layouts, every regrouping\n", n_struct, uni.size() - n_struct);
  fflush(stdout);

#pragma omp parallel for schedule(dynamic, 64)
  for (long k = 0; k < (do_unary ? (long)uni.size() : 0); ++k) {
    const Flat& f = uni[(size_t)k];
    unsigned ncuts = 1u << (f.first.size() - 1);
    for (unsigned cuts = 0; cuts < ncuts; ++cuts) check_unary(regroup(f.first, f.second, cuts));
  }

  std::vector<Flat> puni;
  flat_universe(pr, pe, &puni);
  stride_universe(std::min(pr, 2), std::min(pe, 3), 4, &puni);
  std::vector<Layout> pl;
  for (const Flat& f : puni) {
    unsigned ncuts = 1u << (f.first.size() - 1);
    for (unsigned cuts = 0; cuts < ncuts; ++cuts) pl.push_back(regroup(f.first, f.second, cuts));
  }
  printf("pair universe: %zu layouts -> %zu ordered pairs, plus %ld random pairs from the unary universe\n",
         pl.size(), pl.size() * pl.size(), nrandom);
  fflush(stdout);
  const long a_begin = do_pairs ? (long)pl.size() * slice_k / slice_n : 0, a_end = do_pairs ? (long)pl.size() * (slice_k + 1) / slice_n : 0;
#pragma omp parallel for schedule(dynamic, 4)
  for (long a = a_begin; a < a_end; ++a)
    for (size_t b = 0; b < pl.size(); ++b) {
      check_pair(pl[(size_t)a], pl[b]);
      check_tiler(pl[(size_t)a], pl[b]);
    }

  std::vector<std::pair<Layout, Layout>> rnd;
  if (!do_random) nrandom = 0;
  for (long k = 0; k < nrandom; ++k) {
    const Flat& fa = uni[rng() % uni.size()];
    const Flat& fb = uni[rng() % uni.size()];
    rnd.push_back({regroup(fa.first, fa.second, (unsigned)(rng() % (1u << (fa.first.size() - 1)))),
                   regroup(fb.first, fb.second, (unsigned)(rng() % (1u << (fb.first.size() - 1))))});
  }
#pragma omp parallel for schedule(dynamic, 64)
  for (long k = 0; k < nrandom; ++k) {
    check_pair(rnd[(size_t)k].first, rnd[(size_t)k].second);
    check_tiler(rnd[(size_t)k].first, rnd[(size_t)k].second);
  }

  long failures = 0;
  for (auto& kv : tallies) {
    printf("%-40s cases %10ld  checked-ok %10ld  failed %ld\n", kv.first.c_str(), kv.second.cases.load(), kv.second.ok.load(),
           kv.second.fail.load());
    if (kv.second.fail.load()) printf("    first failure: %s\n", kv.second.first_failure.c_str());
    failures += kv.second.fail.load();
  }
  printf(failures ? "FAILED\n" : "ALL POST-CONDITIONS HOLD\n");
  return failures ? 1 : 0;
}
