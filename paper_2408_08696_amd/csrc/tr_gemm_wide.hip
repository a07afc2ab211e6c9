// Projection GEMM for prompt ingestion: y[n, O] = a[n, K] * w[O, K]^T with n up to WIDE_MAX_ROWS rows at once.
//
// The decode-step kernel (tr_gemm_mfma.hip) reads every weight byte once per 128 rows at most, so a prompt of
// 512 tokens streams the model four times.  Here a workgroup of eight waves owns NW consecutive out-tiles and a
// block of 8 * RTW row tiles (each wave RTW tiles of 16 rows); with RTW = 4 one workgroup spans all 512 rows and
// the weights are read from memory exactly once per pass.  Where several row blocks share an out-tile group,
// their workgroups have linear ids congruent modulo 8, land on one XCD, and share the group's weights through
// that XCD's L2.
//
// Weight tiles travel global -> registers -> LDS, loaded cooperatively by all eight waves 24 tiles at a time
// (24 / NW k-steps) into a double buffer (one workgroup barrier per stage) with two further stages in flight in
// registers.  Every wave multiplies each weight tile it reads from LDS with its RTW activation tiles (global ->
// registers, prefetched four k-steps deep).  A wave ends with the sums over its k range for its rows: no
// cross-wave reduction, the epilogue runs from registers.  Projections with few out-tiles (o and down) are split
// over k so that the launch still fills the chip; the residual kernel adds the partial sums.
//
// What bounds it (7B gate/up projection of 511 rows, 92 Gflop): with one row tile per wave the LDS set the pace
// (every MFMA needs a 1 KiB tile read, the LDS delivers one per 8 clocks to the whole compute unit): 109 us.
// With two or four row tiles per wave, 86-94 us = 1.0 PFLOP/s at a shader clock of 1.85 GHz (measured during the
// launch), the matrix pipe 68 % busy.  That time did not move with the MFMA shape, the depth of the LDS read-ahead,
// the place of the LDS hand-over in the stage, the stage size, a second workgroup per compute unit, or weight
// stages brought in by direct global -> LDS loads; it follows the volume of global loads a compute unit issues
// (-33 % without the weight loads, -15 % with one activation tile for all waves), 19-24 bytes per clock against
// 60 for a loop of nothing but loads: the waves that load are the waves that must keep the matrix pipe fed, they
// issue in order, and a load that waits for a slot in the memory pipe holds up the MFMAs behind it.
//
// Same packed weight layout, fragment-ordered activations and epilogues (plain store, RoPE + cache append,
// SwiGLU) as the decode kernel.
#include "tr_kernels.h"

namespace tr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ inline f32x16 mfma32w(const u32x4 &a, const u32x4 &b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

constexpr int WIDE_WAVES = 8;
constexpr int WIDE_TPS = 24;                    // weight tiles per LDS stage (24 KiB)
constexpr int WIDE_TPW = WIDE_TPS / WIDE_WAVES; // tiles a wave loads per stage
constexpr int WIDE_PA = 4;                      // k-steps of activation tiles a wave keeps in flight

// NW: out-tiles per workgroup (SwiGLU: NW / 2 gate + NW / 2 up); RTW: row tiles per wave.
template <int MODE, bool SCALED, int NW, int RTW>
__global__ __launch_bounds__(WIDE_WAVES * 64) void k_gemm_wide(GemmArgs g, int32_t row_tiles) {
  constexpr int KS = WIDE_TPS / NW; // k-steps per stage
  constexpr int P = MODE == GEMM_SWIGLU ? NW / 2 : NW;
  static_assert(KS * NW == WIDE_TPS && (KS == 2 || KS == 4), "a pass over the activation registers is 1 or 2 stages");
  __shared__ u32x4 buf[2][WIDE_TPS][64]; // 48 KiB
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // in a scalar register: what depends on it alone is uniform
  const int KT = g.K / 32;
  // linear id -> (k-split, out-tile group, row block): ids that differ by 8 share an XCD, so the row blocks of
  // a group are 8 apart; groups are numbered (id % 8) + 8 * (id / (8 * row_blocks))
  const int row_blocks = (row_tiles + WIDE_WAVES * RTW - 1) / (WIDE_WAVES * RTW);
  const int per_split = ((g.groups + 7) / 8) * 8 * row_blocks;
  const int split = blockIdx.x / per_split, id = blockIdx.x - split * per_split;
  const int bx = (id & 7) + 8 * (id / (8 * row_blocks));
  const int rb = (id >> 3) % row_blocks;
  if (bx >= g.groups) return; // uniform over the workgroup (group count not a multiple of 8)
  // this split's k-steps [k0, k1): equal shares rounded up to whole stages
  int per_k = (KT + g.splits - 1) / g.splits;
  per_k = (per_k + KS - 1) / KS * KS;
  const int k0 = split * per_k, k1 = k0 + per_k < KT ? k0 + per_k : KT;
  const int tile0 = bx * g.part_q + (bx < g.part_rem ? bx : g.part_rem);
  const int n_valid = g.part_q + (bx < g.part_rem ? 1 : 0);

  // the WIDE_TPW weight tiles of a stage this wave fetches: stage tile j = wave + 8 i is (k-step j / NW, tile j % NW)
  const u32x4 *wsrc[WIDE_TPW];
  int wk[WIDE_TPW];
#pragma unroll
  for (int i = 0; i < WIDE_TPW; ++i) {
    const int j = wave + WIDE_WAVES * i, u = j % NW;
    wk[i] = j / NW;
    const int uu = u < P ? u : u - P;   // SwiGLU: tiles P .. 2P-1 come from the up matrix
    int t = tile0 + (uu < n_valid ? uu : 0);
    int sidx = 0;
    while (sidx + 1 < g.n_seg && t >= g.seg[sidx].out_tiles) {
      t -= g.seg[sidx].out_tiles;
      ++sidx;
    }
    const bf16_t *mat = (MODE == GEMM_SWIGLU && u >= P) ? g.w2 : g.seg[sidx].w;
    wsrc[i] = reinterpret_cast<const u32x4 *>(mat) + (size_t)t * KT * 64 + lane;
  }
  const int n_stages = (k1 - k0 + KS - 1) / KS;
  u32x4 wreg[2][WIDE_TPW]; // two weight stages in flight in registers
  auto load_stage = [&](int slot, int s) { // unconditional, clamped: the counts in flight stay compile-time facts
#pragma unroll
    for (int i = 0; i < WIDE_TPW; ++i) {
      int kt = k0 + s * KS + wk[i];
      kt = kt < k1 ? kt : k1 - 1;
      wreg[slot][i] = __builtin_nontemporal_load(wsrc[i] + (size_t)kt * 64);
    }
  };
  // tiles of k-steps past the end of the k range go to LDS as zeros, so the multiply loop needs no tail case
  auto store_stage = [&](int slot, int b, int s) {
#pragma unroll
    for (int i = 0; i < WIDE_TPW; ++i) {
      const bool in_range = k0 + s * KS + wk[i] < k1;
      buf[b][wave + WIDE_WAVES * i][lane] = in_range ? wreg[slot][i] : u32x4{0u, 0u, 0u, 0u};
    }
  };

  // MFMA shape: v_mfma_f32_32x32x16_bf16 (same rate per flop as the 16x16x32 form, half as many instructions and
  // LDS reads per flop).  Its operands are rebuilt from the 16x32 fragment tiles by addressing
  // alone: for k-half h of a k-step, lane l supplies 8 k-values 16 h + 8 (l / 32) .. + 7 of item l % 32, i.e.
  // lane slot (l % 16) + 16 (2 h + l / 32) of the first (l % 32 < 16) or second tile of a pair.  A weight pair
  // is out-tiles (2p, 2p + 1), or for SwiGLU (gate tile p, up tile p); an activation pair is two consecutive row
  // tiles.  The 32 x 32 result leaves lane l with row l % 32 of the row pair and, in elements 4q .. 4q + 3,
  // features 8 q + 4 (l / 32) .. + 3 of the 32 the weight pair spans.
  constexpr int NP2 = NW / 2, RP2 = RTW / 2;
  static_assert(NW % 2 == 0 && RTW % 2 == 0, "tiles are consumed in pairs");
  const int half_sel = (lane >> 4) & 1, hb = lane >> 5;
  const int frag_slot = (lane & 15) + 16 * hb; // + 32 for the second k-half

  // this wave's row tiles rt0 .. rt0 + RTW - 1; a short last block leaves some of them, or whole waves, without
  // rows: those multiply the last tile again and store nothing
  const int rt0 = (rb * WIDE_WAVES + wave) * RTW;
  const bool wave_live = rt0 < row_tiles;
  const u32x4 *abase = reinterpret_cast<const u32x4 *>(g.a_frag);
  int aoff[RP2];
#pragma unroll
  for (int j = 0; j < RP2; ++j) {
    const int rt = rt0 + 2 * j + half_sel;
    aoff[j] = (rt < row_tiles ? rt : row_tiles - 1) * 64 + frag_slot;
  }
  u32x4 aq[WIDE_PA][RP2][2];
  auto issue_a = [&](int slot, int kt) {
    const int kc = kt < k1 ? kt : k1 - 1;
#pragma unroll
    for (int j = 0; j < RP2; ++j) {
      aq[slot][j][0] = abase[(size_t)kc * row_tiles * 64 + aoff[j]];
      aq[slot][j][1] = abase[(size_t)kc * row_tiles * 64 + aoff[j] + 32];
    }
  };
  // LDS tile of pair p that this lane reads, relative to the k-step's first tile
  int wsel[NP2];
#pragma unroll
  for (int p2 = 0; p2 < NP2; ++p2) wsel[p2] = MODE == GEMM_SWIGLU ? p2 + P * half_sel : 2 * p2 + half_sel;

  // register slot of stage s is s & 1; at the top of iteration s the slots hold stages s + 1 and s + 2
  load_stage(0, 0);
#pragma unroll
  for (int j = 0; j < WIDE_PA; ++j) issue_a(j, k0 + j);
  load_stage(1, 1);
  store_stage(0, 0, 0);
  load_stage(0, 2);
  f32x16 acc[NP2][RP2];
#pragma unroll
  for (int u = 0; u < NP2; ++u)
#pragma unroll
    for (int j = 0; j < RP2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[u][j][e] = 0.f;
  __syncthreads();

  for (int s0 = 0; s0 < n_stages; s0 += 2) {
#pragma unroll
    for (int si = 0; si < 2; ++si) { // s & 1 == si: buffer, register slots and activation registers are static
      const int s = s0 + si;
      // the stage's weight pairs in order (k-step, pair), both k-halves of the next pair requested from LDS before
      // the current pair is multiplied, so that a read has the MFMAs of another pair to land behind (two pairs
      // ahead measured no faster)
      u32x4 wc0 = buf[si][wsel[0]][frag_slot], wc1 = buf[si][wsel[0]][frag_slot + 32];
#pragma unroll
      for (int t = 0; t < KS * NP2; ++t) {
        u32x4 wn0 = wc0, wn1 = wc1;
        if (t + 1 < KS * NP2) {
          const int kn = (t + 1) / NP2, pn = (t + 1) % NP2;
          wn0 = buf[si][kn * NW + wsel[pn]][frag_slot];
          wn1 = buf[si][kn * NW + wsel[pn]][frag_slot + 32];
        }
        __builtin_amdgcn_sched_barrier(0); // keep this order: left alone, the scheduler bunches the reads and spills
        const int k = t / NP2, p2 = t % NP2;
        const int slot = (si * KS + k) % WIDE_PA;
#pragma unroll
        for (int j = 0; j < RP2; ++j) acc[p2][j] = mfma32w(wc0, aq[slot][j][0], acc[p2][j]);
#pragma unroll
        for (int j = 0; j < RP2; ++j) acc[p2][j] = mfma32w(wc1, aq[slot][j][1], acc[p2][j]);
        if (p2 + 1 == NP2) issue_a(slot, k0 + s * KS + k + WIDE_PA); // the k-step's activation registers are free
        __builtin_amdgcn_sched_barrier(0);
        wc0 = wn0;
        wc1 = wn1;
      }
      store_stage(si ^ 1, si ^ 1, s + 1); // that buffer was last read before the previous barrier
      load_stage(si ^ 1, s + 3);
      __syncthreads(); // uniform: every wave runs every stage
    }
  }
  if (!wave_live) return;

  // epilogue from registers
#pragma unroll
  for (int j = 0; j < RP2; ++j) {
    const int row = 16 * (rt0 + 2 * j) + (lane & 31);
    const int rt = row >> 4, r = row & 15;
    if (rt >= row_tiles) continue;
    float sc_row = 1.0f;
    if (SCALED) { // per-row RMS scale from n_ssq (<= 8) partial sums of squares; the row's two lanes fetch alternate chunks
      float ss = 0.f;
      if (row < g.n) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (hb + 2 * c < g.n_ssq) ss += g.row_ssq[(size_t)row * g.n_ssq + hb + 2 * c];
      }
      ss += __shfl_xor(ss, 32);
      sc_row = 1.0f / sqrtf(ss / (float)g.norm_dim + g.eps);
    }
#pragma unroll
    for (int p2 = 0; p2 < NP2; ++p2) {
#pragma unroll
      for (int q = 0; q < (MODE == GEMM_SWIGLU ? 2 : 4); ++q) {
        // STORE: elements 4q .. 4q+3 are features 8 (q & 1) + 4 hb .. + 3 of out-tile 2 p2 + q / 2
        // SWIGLU: elements 4q .. (gate) and 8 + 4q .. (up) are features 8 q + 4 hb .. + 3 of tile p2
        const int u = MODE == GEMM_SWIGLU ? p2 : 2 * p2 + (q >> 1);
        if (u >= n_valid) continue;
        const int o = (tile0 + u) * 16 + 8 * (MODE == GEMM_SWIGLU ? q : (q & 1)) + 4 * hb;
        const f32x16 &a = acc[p2][j];
        if (MODE == GEMM_STORE) {
          if (row >= g.n) continue;
          const f32x4 v = f32x4{a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]} * sc_row;
          if (g.rope.q == nullptr) {
            *reinterpret_cast<float4 *>(g.y + (size_t)split * g.split_stride + (size_t)row * g.ldy + o) =
                float4{v[0], v[1], v[2], v[3]};
          } else {
            // fused Q/K/V epilogue, as in the decode kernel: (o, o+1) and (o+2, o+3) are rotation pairs
            const GemmRope &rp = g.rope;
            const int hd = rp.hd, head = o / hd, dd = o - head * hd;
            const int pos = *rp.d_len + row;
            float a0 = v[0], b0 = v[1], a1 = v[2], b1 = v[3];
            if (head < rp.H + rp.Hkv) {
              const float *cs = rp.rope + (size_t)row * hd + (dd >> 1);
              const float c0 = cs[0], c1 = cs[1], s0 = cs[hd / 2], s1 = cs[hd / 2 + 1];
              a0 = v[0] * c0 - v[1] * s0; b0 = v[1] * c0 + v[0] * s0;
              a1 = v[2] * c1 - v[3] * s1; b1 = v[3] * c1 + v[2] * s1;
            }
            const bf16_t e0 = f32_to_bf16(a0), e1 = f32_to_bf16(b0), e2 = f32_to_bf16(a1), e3 = f32_to_bf16(b1);
            if (head < rp.H + rp.Hkv) {
              bf16_t *dst;
              if (head < rp.H) dst = rp.q + ((size_t)row * rp.H + head) * hd + dd;
              else if (rp.tiled) dst = rp.k_layer + (size_t)(head - rp.H) * rp.cap * hd + kv_k_index(pos, dd);
              else dst = rp.k_layer + ((size_t)(head - rp.H) * rp.cap + pos) * hd + dd;
              *reinterpret_cast<ushort4 *>(dst) = ushort4{e0, e1, e2, e3};
            } else {
              bf16_t *dst = rp.v_layer + (size_t)(head - rp.H - rp.Hkv) * hd * rp.cap;
              if (rp.tiled) {
                dst[kv_v_index(pos, dd)] = e0; dst[kv_v_index(pos, dd + 1)] = e1;
                dst[kv_v_index(pos, dd + 2)] = e2; dst[kv_v_index(pos, dd + 3)] = e3;
              } else {
                dst[(size_t)dd * rp.cap + pos] = e0; dst[(size_t)(dd + 1) * rp.cap + pos] = e1;
                dst[(size_t)(dd + 2) * rp.cap + pos] = e2; dst[(size_t)(dd + 3) * rp.cap + pos] = e3;
              }
            }
          }
        } else {
          // h[row, o .. o+3] = bf16(silu(gate) * up) in fragment order over all row tiles; rows past n are zeros
          const bool live = row < g.n;
          const f32x4 gt = f32x4{a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]} * sc_row;
          const f32x4 up = f32x4{a[8 + 4 * q], a[9 + 4 * q], a[10 + 4 * q], a[11 + 4 * q]} * sc_row;
          ushort4 hv;
          hv.x = live ? f32_to_bf16(gt[0] / (1.0f + __expf(-gt[0])) * up[0]) : (bf16_t)0;
          hv.y = live ? f32_to_bf16(gt[1] / (1.0f + __expf(-gt[1])) * up[1]) : (bf16_t)0;
          hv.z = live ? f32_to_bf16(gt[2] / (1.0f + __expf(-gt[2])) * up[2]) : (bf16_t)0;
          hv.w = live ? f32_to_bf16(gt[3] / (1.0f + __expf(-gt[3])) * up[3]) : (bf16_t)0;
          const size_t fslot = ((size_t)(o >> 5) * row_tiles + rt) * 64 + r + 16 * ((o & 31) >> 3);
          store_stream(g.h_frag + fslot * 8 + (o & 7), hv);
        }
      }
    }
  }
}

bool gemm_wide_supported(int32_t n, int32_t K, int32_t O) {
  return n >= 1 && n <= WIDE_MAX_ROWS && K % 32 == 0 && K >= 64 && O % 32 == 0;
}

template <int NW, int RTW>
static hipError_t launch_shape(const GemmArgs &g, int row_tiles, unsigned grid, hipStream_t st, KernelTimer tm) {
  const dim3 block(WIDE_WAVES * 64);
  if (g.mode == GEMM_SWIGLU) {
    if (g.row_ssq != nullptr) return launch(k_gemm_wide<GEMM_SWIGLU, true, NW, RTW>, dim3(grid), block, 0, st, tm, g, row_tiles);
    return launch(k_gemm_wide<GEMM_SWIGLU, false, NW, RTW>, dim3(grid), block, 0, st, tm, g, row_tiles);
  }
  if (g.row_ssq != nullptr) return launch(k_gemm_wide<GEMM_STORE, true, NW, RTW>, dim3(grid), block, 0, st, tm, g, row_tiles);
  return launch(k_gemm_wide<GEMM_STORE, false, NW, RTW>, dim3(grid), block, 0, st, tm, g, row_tiles);
}

// Chooses the workgroup shape, fills the tile assignment and launches.  g.n is the total row count
// (<= WIDE_MAX_ROWS); a_frag / h_frag use ceil(n / 16) row tiles; the RMS scale takes at most 8 partial sums per
// row.  max_splits > 1 (plain store without scale only): y[s] = y + s * split_stride receives the partial sum
// of k-range s, and *out_splits how many the launch used.
//   Shapes: 12 out-tiles x 2 row tiles per wave, 6 x 4 (one workgroup spans 512 rows) or 6 x 2.
hipError_t launch_gemm_wide(const GemmArgs &args, int32_t max_splits, int32_t *out_splits, hipStream_t st, KernelTimer tm) {
  GemmArgs g = args;
  if (g.n < 1 || g.n > WIDE_MAX_ROWS || g.K % 32 != 0 || g.K < 64 || (g.row_ssq != nullptr && g.n_ssq > 8))
    return hipErrorInvalidValue;
  int32_t total = 0;
  for (int i = 0; i < g.n_seg; ++i) total += g.seg[i].out_tiles;
  if (total < 1 || (g.mode != GEMM_STORE && g.mode != GEMM_SWIGLU)) return hipErrorInvalidValue;
  const bool may_split = g.mode == GEMM_STORE && g.rope.q == nullptr && g.row_ssq == nullptr && max_splits > 1;
  const int row_tiles = (g.n + 15) / 16;
  const int unit = g.mode == GEMM_SWIGLU ? 2 : 1; // a gate/up pair occupies two of the NW tiles
  auto groups_of = [&](int nw) { return (total + nw / unit - 1) / (nw / unit); };
  // Shape and K-splits by a cost model of what bounds the kernel, the KiB a workgroup pulls per k-step (its row
  // tiles and its weight tiles, 1 KiB each) times its k-steps, per round of 256 workgroups, plus a fixed cost
  // per round (ramp and epilogue, in the same unit) and what the partial sums of a K-split cost to write and
  // re-read.
  const int KT = g.K / 32;
  int nw = 12, rtw = 2, best_splits = 1;
  double best = 1e30;
  static const int cand[3][2] = {{12, 2}, {6, 4}, {6, 2}};
  for (int c = 0; c < 3; ++c) {
    const int cnw = cand[c][0], crtw = cand[c][1], ks = WIDE_TPS / cnw;
    if (row_tiles <= 16 && crtw == 4) continue;
    const int rb = (row_tiles + WIDE_WAVES * crtw - 1) / (WIDE_WAVES * crtw);
    const int rows_wg = row_tiles < WIDE_WAVES * crtw ? row_tiles : WIDE_WAVES * crtw;
    for (int sp = 1; sp <= (may_split ? max_splits : 1); ++sp) {
      int per_k = (KT + sp - 1) / sp;
      per_k = (per_k + ks - 1) / ks * ks;
      if (sp > 1 && (per_k < 8 * ks || (sp - 1) * per_k >= KT)) continue; // at least 8 stages, no empty share
      const int wgs = groups_of(cnw) * rb * sp;
      const int rounds = (wgs + 255) / 256;
      double cost = rounds * ((double)per_k * (rows_wg + cnw) + 150.0);
      if (sp > 1) cost += sp * 160.0 * row_tiles / 32.0;
      if (cost < best) {
        best = cost;
        nw = cnw;
        rtw = crtw;
        best_splits = sp;
      }
    }
  }
  const int row_blocks = (row_tiles + WIDE_WAVES * rtw - 1) / (WIDE_WAVES * rtw);
  g.total_tiles = total;
  g.tiles_per_wg = nw / unit;
  g.groups = groups_of(nw);
  g.part_q = total / g.groups;
  g.part_rem = total % g.groups;
  g.splits = best_splits;
  if (out_splits != nullptr) *out_splits = g.splits;
  const unsigned grid = (unsigned)(((g.groups + 7) / 8) * 8 * row_blocks * g.splits);
  if (nw == 12) return launch_shape<12, 2>(g, row_tiles, grid, st, tm);
  if (rtw == 2) return launch_shape<6, 2>(g, row_tiles, grid, st, tm);
  return launch_shape<6, 4>(g, row_tiles, grid, st, tm);
}

} // namespace tr
