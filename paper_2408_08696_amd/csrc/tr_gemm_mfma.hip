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
// Mapping.  One workgroup owns OT consecutive out-tiles (16*OT output features) and one of `splits`
// K-ranges; its 8 wavefronts take interleaved k-tiles of that range, keep PF k-steps of loads in flight
// in registers, and reduce through LDS in a fixed binary tree at the end.  splits > 1 writes one partial
// result per split (summed in a fixed order by the consumer), so results are run-to-run deterministic.
#include "tr_kernels.h"

namespace tr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int GEMM_WAVES = 8;
constexpr int GEMM_PF = 4; // k-steps of loads in flight per wave

__device__ inline f32x4 mfma16(const u32x4 &a, const u32x4 &b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------
// one-time repack of a row-major [O, K] bf16 matrix into fragment order
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_pack_weight(const bf16_t *__restrict__ src, int32_t O, int32_t K,
                                                     uint4 *__restrict__ dst) {
  const int KT = K / 32;
  const size_t slot = (size_t)blockIdx.x * 256 + threadIdx.x; // one 16-byte lane slot
  const size_t total = (size_t)(O / 16) * KT * 64;
  if (slot >= total) return;
  const int lane = (int)(slot & 63);
  const size_t tile = slot >> 6;
  const int kt = (int)(tile % KT);
  const int ot = (int)(tile / KT);
  const int row = ot * 16 + (lane & 15);
  const int k = kt * 32 + 8 * (lane >> 4);
  dst[slot] = *reinterpret_cast<const uint4 *>(src + (size_t)row * K + k);
}

hipError_t launch_pack_weight(const bf16_t *src, bf16_t *dst, int32_t O, int32_t K, hipStream_t st) {
  const size_t total = (size_t)(O / 16) * (K / 32) * 64;
  hipLaunchKernelGGL(k_pack_weight, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, O, K,
                     reinterpret_cast<uint4 *>(dst));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// the GEMM
// ---------------------------------------------------------------------------------------------
template <int NT, int OT, int MODE>
__global__ __launch_bounds__(GEMM_WAVES * 64) void k_gemm_mfma(GemmArgs g) {
  // SWIGLU: OT must be 1; "tile 0" is the gate matrix, "tile 1" the up matrix, same out-tile index
  constexpr int NW = MODE == GEMM_SWIGLU ? 2 : OT;
  extern __shared__ float red[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int KT = g.K / 32;

  // which segment (weight matrix) and out-tile does this workgroup own
  int tile0 = blockIdx.x * OT; // global out-tile index across the concatenated segments
  const u32x4 *wbase[NW];
  {
    int t = tile0, sidx = 0;
    while (sidx + 1 < g.n_seg && t >= g.seg[sidx].out_tiles) {
      t -= g.seg[sidx].out_tiles;
      ++sidx;
    }
    const u32x4 *w = reinterpret_cast<const u32x4 *>(g.seg[sidx].w) + (size_t)t * KT * 64 + lane;
    if (MODE == GEMM_SWIGLU) {
      wbase[0] = w;
      wbase[NW - 1] = reinterpret_cast<const u32x4 *>(g.w2) + (size_t)t * KT * 64 + lane;
    } else {
#pragma unroll
      for (int u = 0; u < NW; ++u) wbase[u] = w + (size_t)u * KT * 64;
    }
  }
  const u32x4 *abase = reinterpret_cast<const u32x4 *>(g.a_frag) + lane;

  // this workgroup's K-range and this wave's k-tiles in it: kt = kt0 + wave + 8*i
  const int split = blockIdx.y;
  const int per = (KT + g.splits - 1) / g.splits;
  const int kt0 = split * per;
  const int kt1 = kt0 + per < KT ? kt0 + per : KT;
  const int first = kt0 + wave;
  const int nsteps = first < kt1 ? (kt1 - first + GEMM_WAVES - 1) / GEMM_WAVES : 0;

  f32x4 acc[NW][NT];
#pragma unroll
  for (int u = 0; u < NW; ++u)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  u32x4 wq[GEMM_PF][NW], aq[GEMM_PF][NT];
  auto issue = [&](int stage, int step) {
    const size_t kt = (size_t)(first + step * GEMM_WAVES);
#pragma unroll
    for (int u = 0; u < NW; ++u) wq[stage][u] = __builtin_nontemporal_load(wbase[u] + kt * 64);
#pragma unroll
    for (int t = 0; t < NT; ++t) aq[stage][t] = abase[(kt * NT + t) * 64];
  };
#pragma unroll
  for (int j = 0; j < GEMM_PF; ++j)
    if (j < nsteps) issue(j, j);
  for (int base = 0; base < nsteps; base += GEMM_PF) {
#pragma unroll
    for (int j = 0; j < GEMM_PF; ++j) {
      if (base + j < nsteps) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int u = 0; u < NW; ++u) acc[u][t] = mfma16(wq[j][u], aq[j][t], acc[u][t]);
        if (base + j + GEMM_PF < nsteps) issue(j, base + j + GEMM_PF);
      }
    }
  }

  // cross-wave reduction, a fixed binary tree through LDS: in round h the upper h waves of the
  // surviving 2h publish their accumulators and the lower h add them; wave 0 ends with the sum.
  float4 *red4 = reinterpret_cast<float4 *>(red); // [GEMM_WAVES/2][NW][NT][64]
#pragma unroll
  for (int h = GEMM_WAVES / 2; h >= 1; h >>= 1) {
    if (wave >= h && wave < 2 * h) {
#pragma unroll
      for (int u = 0; u < NW; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          red4[(((wave - h) * NW + u) * NT + t) * 64 + lane] =
              float4{acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]};
    }
    __syncthreads();
    if (wave < h) {
#pragma unroll
      for (int u = 0; u < NW; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const float4 o = red4[((wave * NW + u) * NT + t) * 64 + lane];
          acc[u][t][0] += o.x; acc[u][t][1] += o.y; acc[u][t][2] += o.z; acc[u][t][3] += o.w;
        }
    }
    __syncthreads();
  }
  if (wave != 0) return;
  const int r = lane & 15, gq = lane >> 4;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int row = 16 * t + r;
    if (MODE == GEMM_STORE) {
      if (row >= g.n) continue;
      float *yb = g.y + (size_t)split * g.split_stride + (size_t)row * g.ldy;
#pragma unroll
      for (int u = 0; u < NW; ++u) {
        const int o = (tile0 + u) * 16 + 4 * gq;
        *reinterpret_cast<float4 *>(yb + o) = float4{acc[u][t][0], acc[u][t][1], acc[u][t][2], acc[u][t][3]};
      }
    } else {
      // h[row, o .. o+3] = bf16(silu(gate) * up), written in fragment order over (k = o, NT row tiles);
      // rows past n are written as zeros so the consumer's operand tiles are fully defined
      const f32x4 gt = acc[0][t], up = acc[NW - 1][t];
      const bool live = row < g.n;
      ushort4 hv;
      hv.x = live ? f32_to_bf16(gt[0] / (1.0f + __expf(-gt[0])) * up[0]) : (bf16_t)0;
      hv.y = live ? f32_to_bf16(gt[1] / (1.0f + __expf(-gt[1])) * up[1]) : (bf16_t)0;
      hv.z = live ? f32_to_bf16(gt[2] / (1.0f + __expf(-gt[2])) * up[2]) : (bf16_t)0;
      hv.w = live ? f32_to_bf16(gt[3] / (1.0f + __expf(-gt[3])) * up[3]) : (bf16_t)0;
      const int o = tile0 * 16 + 4 * gq;                 // k index of the consumer
      const size_t slot = ((size_t)(o >> 5) * NT + t) * 64 + r + 16 * ((o & 31) >> 3);
      *reinterpret_cast<ushort4 *>(g.h_frag + slot * 8 + (o & 7)) = hv;
    }
  }
}

bool gemm_mfma_supported(int32_t n, int32_t K, int32_t O) {
  return n >= 1 && n <= TR_MAX_NODES && K % 32 == 0 && O % 32 == 0;
}

template <int NT, int OT, int MODE>
static hipError_t launch_k(const GemmArgs &g, int total_tiles, hipStream_t st) {
  constexpr int NW = MODE == GEMM_SWIGLU ? 2 : OT;
  const size_t smem = (size_t)(GEMM_WAVES / 2) * NW * NT * 64 * 16;
  hipLaunchKernelGGL((k_gemm_mfma<NT, OT, MODE>), dim3(total_tiles / OT, g.splits), dim3(GEMM_WAVES * 64), smem, st, g);
  return hipGetLastError();
}

template <int NT>
static hipError_t launch_nt(const GemmArgs &g, int total_tiles, int ot, hipStream_t st) {
  if (g.mode == GEMM_SWIGLU) return launch_k<NT, 1, GEMM_SWIGLU>(g, total_tiles, st);
  if (ot == 2) return launch_k<NT, 2, GEMM_STORE>(g, total_tiles, st);
  return launch_k<NT, 1, GEMM_STORE>(g, total_tiles, st);
}

hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t st) {
  int total = 0;
  bool even = true;
  for (int i = 0; i < g.n_seg; ++i) {
    total += g.seg[i].out_tiles;
    even = even && (g.seg[i].out_tiles % 2 == 0);
  }
  // two out-tiles per workgroup halve the activation re-reads; keep one when that would leave
  // fewer workgroups than compute units
  const int ot = (g.mode != GEMM_SWIGLU && even && (total / 2) * g.splits >= 256) ? 2 : 1;
  switch ((g.n + 15) / 16) {
  case 1: return launch_nt<1>(g, total, ot, st);
  case 2: return launch_nt<2>(g, total, ot, st);
  case 3: return launch_nt<3>(g, total, ot, st);
  case 4: return launch_nt<4>(g, total, ot, st);
  case 5: return launch_nt<5>(g, total, ot, st);
  case 6: return launch_nt<6>(g, total, ot, st);
  case 7: return launch_nt<7>(g, total, ot, st);
  case 8: return launch_nt<8>(g, total, ot, st);
  }
  return hipErrorInvalidValue;
}

} // namespace tr
