// Host walk of a GEMM plan (a checking device for tests, see gemm_plan.hpp): the kernel's loops over
// workgroups, lanes and k tiles with the same index functions (gemm_params.hpp), every global access
// checked against the buffers, the operand tiles passed through a byte model of LDS, and the matrix
// instruction replaced by its definition taken through the fragments' thread-value layouts.
#include <cmath>
#include <cstring>
#include <vector>

#include "gemm_plan.hpp"

namespace lc {

namespace {

float bf16_to_float(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}
float f16_to_float(uint16_t h) {
  const int sign = h >> 15, exp = (h >> 10) & 31, man = h & 1023;
  float v;
  if (exp == 0) v = std::ldexp((float)man, -24);
  else if (exp == 31) v = man ? NAN : INFINITY;
  else v = std::ldexp((float)(man + 1024), exp - 25);
  return sign ? -v : v;
}

struct Walker {
  const lc_gemm_plan& plan;
  const GemmParams& P;
  const uint16_t* A;
  const uint16_t* B;
  float* C;
  int64_t a_elems, b_elems, c_elems;
  bool ok = true;

  // loads one operand tile of k tile kt into the LDS model, lane by lane
  void stage(const uint16_t* base, int64_t elems, const GemmMode& rmode, const GemmMode& kmode, int32_t load, uint32_t row0, uint32_t extent,
             uint32_t BR, uint32_t kt, unsigned char* tile) {
    if (load == kLoadKDirect) {
      // every lane's 16 bytes land at byte 16 * lane of the 1 KiB its wavefront's instruction i fills
      const uint32_t rows_per_lane = BR / 32;
      for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid)
        for (uint32_t i = 0; i < rows_per_lane; ++i) {
          const uint32_t row = gemm_direct_row(rows_per_lane, tid, i), kv = gemm_direct_kvec(row, tid);
          const int64_t off = (int64_t)gemm_mode_eval(rmode, gemm_clamp_row(load, row0 + row, extent)) + 8u * kv + gemm_mode_eval(kmode, kt * kGemmBK);
          const uint32_t lds_at = ((tid >> 6) * rows_per_lane + i) * 1024u + (tid & 63u) * 16u;
          if (lds_at != gemm_lds_offset(row, kv)) { ok = false; return; }
          if (kt * kGemmBK + 8u * kv >= P.K) {   // past K in a short last k tile: the lane's offset is out of range, zeros arrive
            std::memset(tile + lds_at, 0, 16);
            continue;
          }
          if (off % 8 != 0 || off + 8 > elems || kt * kGemmBK + 8u * kv + 8u > P.K) { ok = false; return; }
          std::memcpy(tile + lds_at, base + off, 16);
        }
      return;
    }
    if (load == kLoadRDirect) {
      // k-major tile: lane l of instruction i of wavefront w fills 16-byte unit (w R + i) 64 + l
      const uint32_t rows_per_lane = BR / 32;
      for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid)
        for (uint32_t i = 0; i < rows_per_lane; ++i) {
          uint32_t k, row;
          gemm_rdirect_unit(BR, rows_per_lane, tid, i, &k, &row);
          const int64_t off = (int64_t)gemm_mode_eval(rmode, gemm_clamp_row(load, row0 + row, extent)) + (int64_t)k * kmode.lead_stride +
                              gemm_mode_eval(kmode, kt * kGemmBK);
          const uint32_t lds_at = ((tid >> 6) * rows_per_lane + i) * 1024u + (tid & 63u) * 16u;
          if (k >= (uint32_t)kGemmBK || row + 8 > BR || lds_at != gemm_rdirect_lds_offset(BR, k, row)) { ok = false; return; }
          if (kt * kGemmBK + k >= P.K) {   // past K in a short last k tile: zeros arrive
            std::memset(tile + lds_at, 0, 16);
            continue;
          }
          // the k row's offset is what the k mode's layout function gives, and the slot is the one fragment reads expect
          if (off % 8 != 0 || off + 8 > elems ||
              (int64_t)k * kmode.lead_stride + gemm_mode_eval(kmode, kt * kGemmBK) != (int64_t)gemm_mode_eval(kmode, kt * kGemmBK + k)) {
            ok = false;
            return;
          }
          std::memcpy(tile + lds_at, base + off, 16);
        }
      return;
    }
    for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid) {
      const uint32_t kv = gemm_lane_kvec(load, tid), k0 = kt * kGemmBK + kv * 8u;
      if (load == kLoadRVec) {
        if (tid >= BR) continue;
        const uint32_t block_row = gemm_lane_row(load, tid, 0);
        uint16_t blk[8][8] = {};   // [k][row]
        if (k0 < P.K) {
          const uint32_t rowoff = gemm_mode_eval(rmode, gemm_clamp_row(load, row0 + block_row, extent));
          const uint32_t koff = gemm_mode_eval(kmode, k0);
          for (uint32_t j = 0; j < 8; ++j) {
            const int64_t off = (int64_t)rowoff + koff + (int64_t)j * kmode.lead_stride;
            if (off % 8 != 0 || off + 8 > elems) { ok = false; return; }
            std::memcpy(blk[j], base + off, 16);
          }
        }
        for (uint32_t i = 0; i < 8; ++i) {
          uint16_t v[8];
          for (uint32_t j = 0; j < 8; ++j) v[j] = blk[j][i];
          std::memcpy(tile + gemm_lds_offset(block_row + i, kv), v, 16);
        }
      } else {
        for (uint32_t i = 0; i < BR / 32; ++i) {
          const uint32_t row = gemm_lane_row(load, tid, i);
          const uint32_t rowoff = gemm_mode_eval(rmode, gemm_clamp_row(load, row0 + row, extent));
          uint16_t v[8] = {};
          if (load == kLoadKVec) {
            if (k0 < P.K) {
              const int64_t off = (int64_t)rowoff + gemm_mode_eval(kmode, k0);
              if (off % 8 != 0 || off + 8 > elems) { ok = false; return; }
              std::memcpy(v, base + off, 16);
            }
          } else {
            for (uint32_t j = 0; j < 8; ++j)
              if (k0 + j < P.K) {
                const int64_t off = (int64_t)rowoff + gemm_mode_eval(kmode, k0 + j);
                if (off >= elems) { ok = false; return; }
                v[j] = base[off];
              }
          }
          std::memcpy(tile + gemm_lds_offset(row, kv), v, 16);
        }
      }
    }
  }

  // What a wavefront's lanes receive for one 32 x 16 fragment (rows row_base .. + 31 of the operand tile, k step kk):
  // out[lane][v], v < 8.  Row-major tiles: one 16-byte read per lane.  k-major tiles: two LDS transpose loads
  // (ds_read_b64_tr_b16), whose definition is applied here to the addresses the lanes present: within each group of
  // 16 lanes, lane i's element e is element i % 4 of the 8 bytes lane 4 e + i / 4 points at.
  void fragment(const unsigned char* tile, int32_t load, uint32_t BR, uint32_t row_base, uint32_t kk, uint16_t (*out)[8]) {
    for (uint32_t lane = 0; lane < 64; ++lane) {
      if (load != kLoadRDirect) {
        std::memcpy(out[lane], tile + gemm_lds_offset(row_base + mfma_ab_row(lane), 2u * kk + mfma_ab_kvec(lane)), 16);
        continue;
      }
      for (uint32_t h = 0; h < 2; ++h)
        for (uint32_t e = 0; e < 4; ++e) {
          const uint32_t src_lane = (lane & ~15u) + 4u * e + (lane & 15u) / 4u;
          const uint32_t at = gemm_rdirect_frag_offset(BR, src_lane, row_base, 16u * kk + 8u * mfma_ab_kvec(src_lane) + 4u * h);
          if (at % 8 != 0 || at + 8 > BR * 128u) { ok = false; return; }
          std::memcpy(&out[lane][4 * h + e], tile + at + 2u * (lane & 3u), 2);
        }
    }
  }
};

}  // namespace

lc_status_t gemm_replay_on_host(const lc_gemm_plan& plan, const uint16_t* a, int64_t a_elems, const uint16_t* b, int64_t b_elems, float* c,
                                int64_t c_elems) {
  if (!a || !b || !c) return LC_ERR_INVALID_ARG;
  if (a_elems < plan.a_cosize || b_elems < plan.b_cosize || c_elems < plan.c_cosize) return LC_ERR_INVALID_ARG;
  const GemmParams& P = plan.params;
  Walker w{plan, P, plan.exchanged ? b : a, plan.exchanged ? a : b, c, plan.exchanged ? b_elems : a_elems,
           plan.exchanged ? a_elems : b_elems, c_elems};
  const uint32_t BM = (uint32_t)plan.tile_m, BN = (uint32_t)plan.tile_n, WMB = BM / 64, WNB = BN / 64;
  if (plan.lds_bytes != (P.a_direct ? 5u * BM * 128u : 2u * (BM + BN) * 128u) || (P.a_direct && BM != BN)) return LC_ERR_INVALID_ARG;
  Layout tv_a, tv_b, tv_c;
  mfma_fragment_layout(0, &tv_a);
  mfma_fragment_layout(1, &tv_b);
  mfma_fragment_layout(2, &tv_c);
  auto to_float = plan.ab_dtype == LC_BF16 ? bf16_to_float : f16_to_float;
  std::vector<unsigned char> lds((BM + BN) * 128u);   // one k tile of A and B is enough for a sequential walk
  std::vector<float> acc((size_t)BM * BN);
  std::vector<char> covered((size_t)P.tiles_m * P.tiles_n, 0);
  const uint32_t n_tiles = P.tiles_m * P.tiles_n;
  const int32_t a_kind = gemm_effective_load(P.a_load, P.a_direct), b_kind = gemm_effective_load(P.b_load, P.b_direct);
  const uint16_t* const a_all = w.A;
  const uint16_t* const b_all = w.B;
  float* const c_all = c;
  const int64_t a_all_elems = w.a_elems, b_all_elems = w.b_elems, c_all_elems = c_elems;
  for (uint32_t batch = 0; batch < P.L; ++batch) {
  // the batch entry's offsets are folded into the three base pointers, as the kernel does with blockIdx.y
  const uint32_t ao = gemm_mode_eval(P.a_l, batch), bo = gemm_mode_eval(P.b_l, batch), co = gemm_mode_eval(P.c_l, batch);
  if (ao > a_all_elems || bo > b_all_elems || co > c_all_elems) return LC_ERR_INVALID_ARG;
  w.A = a_all + ao;
  w.B = b_all + bo;
  w.a_elems = a_all_elems - ao;
  w.b_elems = b_all_elems - bo;
  c = c_all + co;
  c_elems = c_all_elems - co;
  std::fill(covered.begin(), covered.end(), 0);
  for (uint32_t block = 0; block < n_tiles; ++block) {
    uint32_t tm, tn;
    const uint32_t order = gemm_tile_order_of_block(block, n_tiles);
    if (order >= n_tiles) return LC_ERR_INVALID_ARG;
    gemm_tile_of_order(P, order, &tm, &tn);
    if (tm >= P.tiles_m || tn >= P.tiles_n || covered[(size_t)tm * P.tiles_n + tn]) return LC_ERR_INVALID_ARG;   // every tile exactly once
    covered[(size_t)tm * P.tiles_n + tn] = 1;
    const uint32_t m0 = tm * BM, n0 = tn * BN;
    std::fill(acc.begin(), acc.end(), 0.f);
    for (uint32_t kt = 0; kt < P.k_tiles; ++kt) {
      w.stage(w.A, w.a_elems, P.a_r, P.a_k, a_kind, m0, P.M, BM, kt, lds.data());
      w.stage(w.B, w.b_elems, P.b_r, P.b_k, b_kind, n0, P.N, BN, kt, lds.data() + BM * 128u);
      if (!w.ok) return LC_ERR_INVALID_ARG;
      for (uint32_t wave = 0; wave < 4; ++wave) {
        const uint32_t wm = wave & 1u, wn = wave >> 1;
        for (uint32_t kk = 0; kk < kGemmBK / 16; ++kk)
          for (uint32_t i = 0; i < WMB; ++i)
            for (uint32_t j = 0; j < WNB; ++j) {
              // gather the two 32 x 16 fragments from the lanes' LDS reads, through the thread-value layouts
              float fa[32][16], fb[32][16];
              uint16_t va[64][8], vb[64][8];
              w.fragment(lds.data(), a_kind, BM, wm * WMB * 32u + 32u * i, kk, va);
              w.fragment(lds.data() + BM * 128u, b_kind, BN, wn * WNB * 32u + 32u * j, kk, vb);
              if (!w.ok) return LC_ERR_INVALID_ARG;
              for (uint32_t lane = 0; lane < 64; ++lane)
                for (uint32_t v = 0; v < 8; ++v) {
                  const int64_t ca = tv_a((int64_t)lane + 64 * v), cb = tv_b((int64_t)lane + 64 * v);   // row + 32 k
                  fa[ca % 32][ca / 32] = to_float(va[lane][v]);
                  fb[cb % 32][cb / 32] = to_float(vb[lane][v]);
                }
              // D = A B^T + D, then back to the lanes' accumulators through the C fragment layout
              for (uint32_t lane = 0; lane < 64; ++lane)
                for (uint32_t v = 0; v < 16; ++v) {
                  const int64_t cc = tv_c((int64_t)lane + 64 * v);   // m + 32 n
                  const uint32_t r = (uint32_t)(cc % 32), col = (uint32_t)(cc / 32);
                  if (r != mfma_c_row(lane, v) || col != mfma_c_col(lane)) return LC_ERR_INVALID_ARG;
                  float s = 0.f;
                  for (uint32_t k = 0; k < 16; ++k) s += fa[r][k] * fb[col][k];
                  acc[(size_t)(wm * WMB * 32u + 32u * i + r) * BN + (wn * WNB * 32u + 32u * j + col)] += s;
                }
            }
      }
    }
    // epilogue, lane by lane
    for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid) {
      const uint32_t lane = tid & 63u, wave = tid >> 6, wm = wave & 1u, wn = wave >> 1;
      for (uint32_t j = 0; j < WNB; ++j) {
        const uint32_t nl = wn * WNB * 32u + 32u * j + mfma_c_col(lane), n = n0 + nl;
        if (n >= P.N) continue;
        const uint32_t noff = gemm_mode_eval(P.c_n, n);
        for (uint32_t i = 0; i < WMB; ++i)
          for (uint32_t g = 0; g < 4; ++g) {
            const uint32_t ml = wm * WMB * 32u + 32u * i + mfma_c_row(lane, 4u * g), m = m0 + ml;
            if (P.c_vec) {
              if (m >= P.M) continue;
              const int64_t off = (int64_t)gemm_mode_eval(P.c_m, m) + noff;
              if (off % 4 != 0 || off + 4 > c_elems || m + 4 > P.M) return LC_ERR_INVALID_ARG;
              for (uint32_t v = 0; v < 4; ++v) c[off + v] += acc[(size_t)(ml + v) * BN + nl];
            } else {
              for (uint32_t v = 0; v < 4; ++v)
                if (m + v < P.M) {
                  const int64_t off = (int64_t)gemm_mode_eval(P.c_m, m + v) + noff;
                  if (off >= c_elems) return LC_ERR_INVALID_ARG;
                  c[off] += acc[(size_t)(ml + v) * BN + nl];
                }
            }
          }
      }
    }
  }
  }
  return LC_OK;
}

}  // namespace lc
