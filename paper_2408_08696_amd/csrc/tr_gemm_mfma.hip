// Weight-streaming skinny GEMM on the matrix cores: y[n, O] = a[n, K] * w[O, K]^T with n <= 128 rows
// (the tree nodes), bf16 operands, float32 accumulation.  Every weight byte is read from HBM exactly
// once per call; the kernel is bound by that stream, the MFMA work (2*n flop per weight element) only
// has to keep up.
//
// Operand layouts.  v_mfma_f32_16x16x32_bf16 computes D[16 x 16] += A[16 x 32] * B[32 x 16] where lane l
// supplies A[l%16][8*(l/16) .. +7] and B[8*(l/16) .. +7][l%16] as one 16-byte register group, and receives
// D[4*(l/16) .. +3][l%16].  Both operands are therefore stored in memory in "fragment order": a tile of
// 16 rows x 32 k is 1 KiB, lane l's 16 bytes at offset 16*l, so that one wave-wide 16-byte load is one
// fully contiguous KiB and lands directly in MFMA operand registers.
//   weights (packed once by k_pack_weight):   tile (ot, kt) at ((ot * K/32 + kt) * 1 KiB)
//   activations (written so by their producers): tile (kt, nt) at ((kt * NT + nt) * 1 KiB), NT = ceil(n/16)
// With A = weight tile and B = activation tile, lane l ends with outputs o0 + 4*(l/16) .. +3 of row
// 16*nt + l%16.
//
// Mapping.  One workgroup owns up to NW consecutive out-tiles (16*NW output features; the tiles are dealt
// evenly over the workgroups) and one of `splits` K-ranges; its GW = 8 wavefronts (4 in the NW = 8
// variant) take interleaved k-tiles of that range, keep PF k-steps of loads in flight in registers, and
// reduce through LDS at the end, each wave ending up with (and storing) its share of the output tiles.
// splits > 1 writes one partial result per split (summed in a fixed order by the consumer), so results
// are run-to-run deterministic.
//
// Why NW is large.  Every workgroup reads the whole activation block of its K-range from L2 (16*NT rows),
// so L2 carries (1 + 16*NT / (16*NW)) bytes per weight byte; measured L2->CU throughput on MI355X is only
// about twice the HBM rate, so the kernel stays HBM-bound only while NW >= NT.  gemm_choose picks
// (NW, workgroups, splits) from a cost model of exactly this trade, close to one workgroup per compute
// unit with NW as large as the register file allows.
//
// Epilogues: plain float32 store (per K-split), gate/up pairs through SwiGLU into the next GEMM's operand
// order, or for the fused Q/K/V projection RoPE plus the query and KV-cache writes (GemmRope).
#include "tr_kernels.h"

namespace tr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int GEMM_WAVES = 8;
// k-steps of loads in flight per wave, bounded by the register file: accumulators take 4*NW*NT VGPRs,
// every stage 4*(NW+NT); 256 VGPRs per wave at two waves per SIMD, about 208 of them usable here
__host__ __device__ constexpr int gemm_pf(int nw, int nt, int waves) {
  // four waves per workgroup leave one wave per SIMD and 512 registers per wave: the accumulators then
  // sit in the upper half of the unified register file and four stages of 4*(8+5) fit the lower half
  const int pf = waves <= 4 ? 4 : (208 - 4 * nw * nt) / (4 * (nw + nt));
  return pf < 1 ? 1 : (pf > 4 ? 4 : pf);
}

__device__ inline f32x4 mfma16(const u32x4 &a, const u32x4 &b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------
// one-time repack of a row-major [O, K] bf16 matrix into fragment order
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pack_weight(const bf16_t *__restrict__ src, int32_t O, int32_t K,
                                                     int32_t rope_hd, uint4 *__restrict__ dst) {
  const int KT = K / 32;
  const size_t slot = (size_t)blockIdx.x * 256 + threadIdx.x; // one 16-byte lane slot
  const size_t total = (size_t)(O / 16) * KT * 64;
  if (slot >= total) return;
  const int lane = (int)(slot & 63);
  const size_t tile = slot >> 6;
  const int kt = (int)(tile % KT);
  const int ot = (int)(tile / KT);
  int row = ot * 16 + (lane & 15);
  if (rope_hd > 0) { // packed row h*hd + 2j + b <- source row h*hd + j + b*hd/2
    const int i = row % rope_hd;
    row = row - i + (i >> 1) + (i & 1) * (rope_hd / 2);
  }
  const int k = kt * 32 + 8 * (lane >> 4);
  dst[slot] = *reinterpret_cast<const uint4 *>(src + (size_t)row * K + k);
}

hipError_t launch_pack_weight(const bf16_t *src, bf16_t *dst, int32_t O, int32_t K, int32_t rope_hd, hipStream_t st) {
  const size_t total = (size_t)(O / 16) * (K / 32) * 64;
  return launch(k_pack_weight, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, KernelTimer{}, src, O, K, rope_hd,
                reinterpret_cast<uint4 *>(dst));
}

// ---------------------------------------------------------------------------------------------
// the GEMM
// ---------------------------------------------------------------------------------------------
// LDS the tail needs: the GW partials of the tiles of one reduce-scatter pass, plus the per-row scales when
// the epilogue applies an RMS scale.  One pass if all tiles fit the 160 KB of a CU, else two (the first
// covers the units of waves 0 .. GW/2-1).
constexpr size_t gemm_scale_lds_bytes(int nt, bool scaled) { return scaled ? (size_t)nt * 16 * sizeof(float) : 0; }
constexpr bool gemm_tail_one_pass(int p, int nt, int mode, int gw, bool scaled) {
  return (size_t)p * nt * (mode == GEMM_SWIGLU ? 2 : 1) * gw * 1024 + gemm_scale_lds_bytes(nt, scaled) <= 160 * 1024;
}
constexpr size_t gemm_tail_red_bytes(int p, int nt, int mode, int gw, bool scaled) {
  const int u = p * nt, upw = (u + gw - 1) / gw;
  const int own0 = gemm_tail_one_pass(p, nt, mode, gw, scaled) ? gw : gw / 2;
  const int units0 = own0 * upw < u ? own0 * upw : u;
  return (size_t)units0 * (mode == GEMM_SWIGLU ? 2 : 1) * gw * 1024;
}

template <int NT, int NW, int MODE, int GW, bool SCALED>
__global__ __launch_bounds__(GW * 64) void k_gemm_mfma(GemmArgs g) {
  // SWIGLU: NW = 2P; weight tiles 0..P-1 come from the gate matrix, P..2P-1 from the up matrix
  constexpr int P = MODE == GEMM_SWIGLU ? NW / 2 : NW; // distinct out-tiles per workgroup
  constexpr int PF = gemm_pf(NW, NT, GW);
  extern __shared__ float red[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int KT = g.K / 32;

  // out-tiles owned by this workgroup: the T tiles are dealt to the G workgroups in contiguous ranges of
  // T/G tiles, the first T%G of them one longer (the host picks G >= T/P, so no range exceeds P).  Tiles
  // are numbered across the concatenated segments (weight matrices) and each looks up its own segment,
  // so a workgroup may straddle two matrices.
  const int bx = blockIdx.x;
  const int tile0 = bx * g.part_q + (bx < g.part_rem ? bx : g.part_rem);
  const int n_valid = g.part_q + (bx < g.part_rem ? 1 : 0);
  const u32x4 *wbase[NW];
#pragma unroll
  for (int u = 0; u < P; ++u) {
    int t = tile0 + (u < n_valid ? u : 0); // unused slots re-read the first tile (a cache hit), never stored
    int sidx = 0;
    while (sidx + 1 < g.n_seg && t >= g.seg[sidx].out_tiles) {
      t -= g.seg[sidx].out_tiles;
      ++sidx;
    }
    wbase[u] = reinterpret_cast<const u32x4 *>(g.seg[sidx].w) + (size_t)t * KT * 64 + lane;
    if (MODE == GEMM_SWIGLU) wbase[P + u] = reinterpret_cast<const u32x4 *>(g.w2) + (size_t)t * KT * 64 + lane;
  }
  const u32x4 *abase = reinterpret_cast<const u32x4 *>(g.a_frag) + lane;

  // this workgroup's K-range and this wave's k-tiles in it: kt = kt0 + wave + 8*i
  const int split = blockIdx.y;
  const int per = (KT + g.splits - 1) / g.splits;
  const int kt0 = split * per;
  const int kt1 = kt0 + per < KT ? kt0 + per : KT;
  const int first = kt0 + wave;
  const int nsteps = first < kt1 ? (kt1 - first + GW - 1) / GW : 0;

  f32x4 acc[NW][NT];
#pragma unroll
  for (int u = 0; u < NW; ++u)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // per-row RMS scale for the epilogue (SCALED kernels, wave 0 only).  Lane group g fetches chunks g and g+4
  // of its row's sums of squares now, with no dependent arithmetic, so the loads retire under the main
  // loop; the tail adds the groups with two shuffles (n_ssq <= 8) and hands the scales out through LDS.
  float row_ss[NT][2];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int row = 16 * t + (lane & 15), c0 = lane >> 4;
    const bool on = SCALED && wave == 0 && row < g.n;
    row_ss[t][0] = on && c0 < g.n_ssq ? g.row_ssq[(size_t)row * g.n_ssq + c0] : 0.f;
    row_ss[t][1] = on && c0 + 4 < g.n_ssq ? g.row_ssq[(size_t)row * g.n_ssq + c0 + 4] : 0.f;
  }

  u32x4 wq[PF][NW], aq[PF][NT];
  auto issue = [&](int stage, int step) {
    const size_t kt = (size_t)(first + step * GW);
#pragma unroll
    for (int u = 0; u < NW; ++u) wq[stage][u] = __builtin_nontemporal_load(wbase[u] + kt * 64);
#pragma unroll
    for (int t = 0; t < NT; ++t) aq[stage][t] = abase[(kt * NT + t) * 64];
  };
#pragma unroll
  for (int j = 0; j < PF; ++j)
    if (j < nsteps) issue(j, j);
  for (int base = 0; base < nsteps; base += PF) {
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      if (base + j < nsteps) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int u = 0; u < NW; ++u) acc[u][t] = mfma16(wq[j][u], aq[j][t], acc[u][t]);
        if (base + j + PF < nsteps) issue(j, base + j + PF);
      }
    }
  }

  // Cross-wave reduction as a reduce-scatter through LDS, then a distributed epilogue.  The NW*NT
  // accumulator tiles form U units of TPU tiles (one tile; for SWIGLU a gate tile and its up tile); wave w
  // owns units w*UPW .. w*UPW+UPW-1.  Every wave publishes its partial of each tile and the owner adds the
  // GW partials in wave order (a fixed order: results are run-to-run identical).  When the GW partials of
  // all tiles fit LDS this is one pass; otherwise two, the first for the units of waves 0 .. GW/2-1.
  // Every wave then scales, activates and stores its own few tiles, instead of one wave storing them all.
  constexpr int TPU = MODE == GEMM_SWIGLU ? 2 : 1;
  constexpr int U = P * NT;
  constexpr int UPW = (U + GW - 1) / GW;
  constexpr int OWN0 = gemm_tail_one_pass(P, NT, MODE, GW, SCALED) ? GW : GW / 2; // waves 0 .. OWN0-1 own pass 0
  float4 *red4 = reinterpret_cast<float4 *>(red); // [unit slot * TPU + k][GW][64]
  float *sc_lds = red + gemm_tail_red_bytes(P, NT, MODE, GW, SCALED) / sizeof(float); // [NT * 16], SCALED only
  if (SCALED && wave == 0) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float ss = row_ss[t][0] + row_ss[t][1];
      ss += __shfl_xor(ss, 16);
      ss += __shfl_xor(ss, 32);
      if (lane < 16) sc_lds[16 * t + lane] = 1.0f / sqrtf(ss / (float)g.norm_dim + g.eps);
    }
  }
  f32x4 fin[UPW][TPU];
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    if (pass == 1 && OWN0 * UPW >= U) break; // every unit was owned by a pass-0 wave
#pragma unroll
    for (int u = 0; u < P; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int id = u * NT + t;
        if ((id / UPW >= OWN0) != (pass == 1)) continue;
        const int slot = (id - pass * OWN0 * UPW) * TPU;
        red4[((size_t)slot * GW + wave) * 64 + lane] = float4{acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]};
        if (MODE == GEMM_SWIGLU)
          red4[((size_t)(slot + 1) * GW + wave) * 64 + lane] =
              float4{acc[P + u][t][0], acc[P + u][t][1], acc[P + u][t][2], acc[P + u][t][3]};
      }
    __syncthreads();
    if ((wave >= OWN0) == (pass == 1)) {
#pragma unroll
      for (int i = 0; i < UPW; ++i) {
        const int id = wave * UPW + i;
#pragma unroll
        for (int k = 0; k < TPU; ++k) {
          f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
          if (id < U) {
            const float4 *src = red4 + ((size_t)((id - pass * OWN0 * UPW) * TPU + k) * GW) * 64 + lane;
#pragma unroll
            for (int w = 0; w < GW; ++w) {
              const float4 o = src[w * 64];
              sum[0] += o.x; sum[1] += o.y; sum[2] += o.z; sum[3] += o.w;
            }
          }
          fin[i][k] = sum;
        }
      }
    }
    if (pass == 0 && OWN0 * UPW < U) __syncthreads(); // pass 1 reuses the buffer
  }

  const int r = lane & 15, gq = lane >> 4;
#pragma unroll
  for (int i = 0; i < UPW; ++i) {
    const int id = wave * UPW + i;
    if (id >= U) continue;
    const int u = id / NT, t = id - u * NT;
    if (u >= n_valid) continue;
    const int row = 16 * t + r;
    const float sc_row = SCALED ? sc_lds[row] : 1.0f;
    const int o = (tile0 + u) * 16 + 4 * gq;
    if (MODE == GEMM_STORE) {
      if (row >= g.n) continue;
      const f32x4 v = f32x4{fin[i][0][0] * sc_row, fin[i][0][1] * sc_row, fin[i][0][2] * sc_row, fin[i][0][3] * sc_row};
      if (g.rope.q == nullptr) {
        float *yb = g.y + (size_t)split * g.split_stride + (size_t)row * g.ldy;
        *reinterpret_cast<float4 *>(yb + o) = float4{v[0], v[1], v[2], v[3]};
      } else {
        // fused Q/K/V epilogue: features o .. o+3 of the concatenated [q | k | v] outputs, in the
        // interleaved order of the packed wq / wk rows: (o, o+1) and (o+2, o+3) are rotation pairs
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
      // h[row, o .. o+3] = bf16(silu(gate) * up), written in fragment order over (k = o, NT row tiles);
      // rows past n are written as zeros so the consumer's operand tiles are fully defined
      const bool live = row < g.n;
      const f32x4 gt = f32x4{fin[i][0][0] * sc_row, fin[i][0][1] * sc_row, fin[i][0][2] * sc_row, fin[i][0][3] * sc_row};
      const f32x4 up = f32x4{fin[i][TPU - 1][0] * sc_row, fin[i][TPU - 1][1] * sc_row, fin[i][TPU - 1][2] * sc_row, fin[i][TPU - 1][3] * sc_row};
      ushort4 hv;
      hv.x = live ? f32_to_bf16(gt[0] / (1.0f + __expf(-gt[0])) * up[0]) : (bf16_t)0;
      hv.y = live ? f32_to_bf16(gt[1] / (1.0f + __expf(-gt[1])) * up[1]) : (bf16_t)0;
      hv.z = live ? f32_to_bf16(gt[2] / (1.0f + __expf(-gt[2])) * up[2]) : (bf16_t)0;
      hv.w = live ? f32_to_bf16(gt[3] / (1.0f + __expf(-gt[3])) * up[3]) : (bf16_t)0;
      const size_t slot = ((size_t)(o >> 5) * NT + t) * 64 + r + 16 * ((o & 31) >> 3);
      store_stream(g.h_frag + slot * 8 + (o & 7), hv);
    }
  }
}

bool gemm_mfma_supported(int32_t n, int32_t K, int32_t O) {
  return n >= 1 && n <= TR_MAX_NODES && K % 32 == 0 && O % 32 == 0;
}

// Kernel variants: (P out-tiles per workgroup, waves).  Accumulators take 4*P*NT registers (twice that
// for SWIGLU pairs), so the larger ones exist only for few row tiles; 8 weight tiles need the four-wave
// form, whose accumulators live in the upper half of the unified register file.
static bool variant_ok(int NT, int p, bool swiglu) {
  const int wt = swiglu ? 2 * p : p;
  if (wt == 8) return NT == 4 || NT == 5;
  if (wt == 6) return true; // eight waves up to 5 row tiles, the four-wave form beyond
  if (wt == 5) return !swiglu && NT <= 5;
  if (swiglu) return wt == 2 || wt == 4;
  return wt >= 1 && wt <= 4;
}

// Pick (P, workgroups per K-split, K-splits).  About max(ceil(T/P), min(T, 256/S)) workgroups share the T
// out-tiles evenly.  The estimate is the slowest workgroup's time in each round of 256 workgroups: the
// KiB it pulls through L2 (its weight tiles once, the activation block of its K-range once) at the
// per-CU rate, or the round's weight stream at the HBM rate if that is slower, plus a fixed cost per
// round and what the consumer pays to re-read K-split partial sums.  Rates in KiB/us, fitted to
// measurements on MI355X.
void gemm_choose(int32_t n, int32_t K, int32_t total_tiles, bool swiglu, int32_t max_splits, int32_t *out_p,
                 int32_t *out_groups, int32_t *out_splits) {
  const int NT = (n + 15) / 16, KT = K / 32;
  const double wmul = swiglu ? 2.0 : 1.0;
  static const int cand[] = {1, 2, 3, 4, 5, 6, 8};
  double best = 1e30;
  int bp = swiglu ? 1 : 1, bg = total_tiles, bs = 1;
  for (int ci = 0; ci < 7; ++ci) {
    const int p = cand[ci];
    if (!variant_ok(NT, p, swiglu)) continue;
    for (int s = 1; s <= max_splits; s *= 2) {
      if (KT / s < GEMM_WAVES) break;
      int groups = 256 / s < total_tiles ? 256 / s : total_tiles;
      if (groups * p < total_tiles) groups = (total_tiles + p - 1) / p;
      const int tpw = (total_tiles + groups - 1) / groups;
      groups = (total_tiles + tpw - 1) / tpw; // fewest workgroups with the same largest share
      const int rounds = (groups * s + 255) / 256;
      const double kts = (double)((KT + s - 1) / s);
      const double l2_kib = kts * (tpw * wmul + NT);
      const double hbm_kib = kts * tpw * wmul * (groups * s < 256 ? groups * s : 256);
      double t = l2_kib / 48.0;
      if (hbm_kib / 6000.0 > t) t = hbm_kib / 6000.0;
      t = rounds * (t + 3.0) + 3.0;
      if (s > 1) t += 2.0 * (s - 1) * NT * total_tiles / 8000.0 + 0.5; // extra KiB of partials written and re-read
      if (t < best) {
        best = t;
        bp = p;
        bg = groups;
        bs = s;
      }
    }
  }
  *out_p = bp;
  *out_groups = bg;
  *out_splits = bs;
}

template <int NT, int P, int MODE, int GW, bool SCALED>
static hipError_t launch_ks(const GemmArgs &g, hipStream_t st, KernelTimer tm) {
  constexpr int NW = MODE == GEMM_SWIGLU ? 2 * P : P;
  const size_t smem = gemm_tail_red_bytes(P, NT, MODE, GW, SCALED) + gemm_scale_lds_bytes(NT, SCALED);
  if (smem > 65536) {
    static bool once = [] {
      return hipFuncSetAttribute(reinterpret_cast<const void *>(&k_gemm_mfma<NT, NW, MODE, GW, SCALED>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) == hipSuccess;
    }();
    if (!once) return hipErrorInvalidValue;
  }
  return launch(k_gemm_mfma<NT, NW, MODE, GW, SCALED>, dim3(g.groups, g.splits), dim3(GW * 64), smem, st, tm, g);
}
// the epilogue's RMS scale is a compile-time property: without it the tail needs no scale hand-out and
// the whole of LDS can hold partial tiles
template <int NT, int P, int MODE, int GW = GEMM_WAVES>
static hipError_t launch_k(const GemmArgs &g, hipStream_t st, KernelTimer tm) {
  if (g.row_ssq != nullptr) return launch_ks<NT, P, MODE, GW, true>(g, st, tm);
  return launch_ks<NT, P, MODE, GW, false>(g, st, tm);
}

template <int NT>
static hipError_t launch_nt(const GemmArgs &g, hipStream_t st, KernelTimer tm) {
  const int p = g.tiles_per_wg;
  const bool swiglu = g.mode == GEMM_SWIGLU;
  if (!variant_ok(NT, p, swiglu) || g.groups < 1 || g.groups > g.total_tiles ||
      (int64_t)g.groups * p < g.total_tiles)
    return hipErrorInvalidValue;
  if (swiglu) {
    if constexpr (NT == 4 || NT == 5) {
      if (p == 4) return launch_k<NT, 4, GEMM_SWIGLU, 4>(g, st, tm);
    }
    if constexpr (NT <= 5) {
      if (p == 3) return launch_k<NT, 3, GEMM_SWIGLU>(g, st, tm);
    } else {
      if (p == 3) return launch_k<NT, 3, GEMM_SWIGLU, 4>(g, st, tm);
    }
    if (p == 2) return launch_k<NT, 2, GEMM_SWIGLU>(g, st, tm);
    if (p == 1) return launch_k<NT, 1, GEMM_SWIGLU>(g, st, tm);
    return hipErrorInvalidValue;
  }
  if constexpr (NT == 4 || NT == 5) {
    if (p == 8) return launch_k<NT, 8, GEMM_STORE, 4>(g, st, tm);
  }
  if constexpr (NT <= 5) {
    if (p == 6) return launch_k<NT, 6, GEMM_STORE>(g, st, tm);
  } else {
    if (p == 6) return launch_k<NT, 6, GEMM_STORE, 4>(g, st, tm);
  }
  if constexpr (NT <= 5) {
    if (p == 5) return launch_k<NT, 5, GEMM_STORE>(g, st, tm);
  }
  switch (p) {
  case 1: return launch_k<NT, 1, GEMM_STORE>(g, st, tm);
  case 2: return launch_k<NT, 2, GEMM_STORE>(g, st, tm);
  case 3: return launch_k<NT, 3, GEMM_STORE>(g, st, tm);
  case 4: return launch_k<NT, 4, GEMM_STORE>(g, st, tm);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_mfma(const GemmArgs &args, hipStream_t st, KernelTimer tm) {
  if (args.groups < 1 || args.total_tiles < 1) return hipErrorInvalidValue;
  GemmArgs g = args;
  g.part_q = g.total_tiles / g.groups;
  g.part_rem = g.total_tiles % g.groups;
  switch ((g.n + 15) / 16) {
  case 1: return launch_nt<1>(g, st, tm);
  case 2: return launch_nt<2>(g, st, tm);
  case 3: return launch_nt<3>(g, st, tm);
  case 4: return launch_nt<4>(g, st, tm);
  case 5: return launch_nt<5>(g, st, tm);
  case 6: return launch_nt<6>(g, st, tm);
  case 7: return launch_nt<7>(g, st, tm);
  case 8: return launch_nt<8>(g, st, tm);
  }
  return hipErrorInvalidValue;
}

} // namespace tr
