// Weight-streaming skinny GEMM on the matrix cores: y[n, O] = a[n, K] * w[O, K]^T, n <= 128 rows
// (the tree nodes), bf16 operands, float32 accumulation.  Every weight byte is read from HBM exactly
// once per call; the kernel is bound by that stream, the MFMA work (2*n flop per weight element)
// only has to keep up.
//
// Mapping.  One workgroup owns 16 output features; its WAVES wavefronts split K between them in
// blocks of 128 and reduce through LDS at the end, so no partial sums ever leave the CU.
// v_mfma_f32_16x16x32_bf16 computes D[16 outs][16 rows] += W[16][32] * A^T[32][16]:
//   lane l holds W[o0 + l%16][8 consecutive k of group l/16]   (A operand)
//        and     A[r0 + l%16][the same 8 k]                    (B operand)
//   D: lane l holds outs o0 + 4*(l/16) .. +3 for row r0 + l%16.
// The contraction index may be permuted freely as long as both operands agree, so within a block
// of 128 k lane group g takes the contiguous 64 bytes k0+32g .. k0+32g+31 (four 16-byte loads that
// feed four MFMA steps): a wave reads 16 rows x 256 contiguous bytes per block from both operands.
#include "tr_kernels.h"

namespace tr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int GEMM_WAVES = 8;
constexpr int GEMM_KB = 128; // k per block

__device__ inline f32x4 mfma16(const uint4 &a, const uint4 &b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int NT, int MODE>
__global__ __launch_bounds__(GEMM_WAVES * 64) void k_gemm_mfma(const bf16_t *__restrict__ a, const bf16_t *__restrict__ w,
                                                               const bf16_t *__restrict__ w2, int32_t n, int32_t K,
                                                               float *__restrict__ y, int32_t ldy,
                                                               bf16_t *__restrict__ hout) {
  constexpr int NW = MODE == GEMM_SWIGLU ? 2 : 1;
  extern __shared__ float red[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int o0 = blockIdx.x * 16;
  const uint4 *wp = reinterpret_cast<const uint4 *>(w + (size_t)(o0 + r) * K + 32 * g);
  const uint4 *wp2 = MODE == GEMM_SWIGLU ? reinterpret_cast<const uint4 *>(w2 + (size_t)(o0 + r) * K + 32 * g) : nullptr;
  const uint4 *ap[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    int row = 16 * t + r;
    row = row < n ? row : n - 1; // rows past n are computed from a valid row and never stored
    ap[t] = reinterpret_cast<const uint4 *>(a + (size_t)row * K + 32 * g);
  }
  f32x4 acc[NW][NT];
#pragma unroll
  for (int u = 0; u < NW; ++u)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[u][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nkb = K / GEMM_KB;
  for (int kb = wave; kb < nkb; kb += GEMM_WAVES) {
    const int off = kb * (GEMM_KB / 8); // in uint4 units
    uint4 wv[NW][4], av[NT][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) wv[0][c] = wp[off + c];
    if (MODE == GEMM_SWIGLU) {
#pragma unroll
      for (int c = 0; c < 4; ++c) wv[NW - 1][c] = wp2[off + c];
    }
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int c = 0; c < 4; ++c) av[t][c] = ap[t][off + c];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int u = 0; u < NW; ++u) acc[u][t] = mfma16(wv[u][c], av[t][c], acc[u][t]);
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
  const int o = o0 + 4 * g;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int row = 16 * t + r;
    if (row >= n) continue;
    if (MODE == GEMM_STORE) {
      *reinterpret_cast<float4 *>(y + (size_t)row * ldy + o) =
          float4{acc[0][t][0], acc[0][t][1], acc[0][t][2], acc[0][t][3]};
    } else if (MODE == GEMM_ADD) {
      float4 *dst = reinterpret_cast<float4 *>(y + (size_t)row * ldy + o);
      float4 cur = *dst;
      cur.x += acc[0][t][0]; cur.y += acc[0][t][1]; cur.z += acc[0][t][2]; cur.w += acc[0][t][3];
      *dst = cur;
    } else {
      const f32x4 gt = acc[0][t], up = acc[NW - 1][t];
      ushort4 hv;
      hv.x = f32_to_bf16(gt[0] / (1.0f + expf(-gt[0])) * up[0]);
      hv.y = f32_to_bf16(gt[1] / (1.0f + expf(-gt[1])) * up[1]);
      hv.z = f32_to_bf16(gt[2] / (1.0f + expf(-gt[2])) * up[2]);
      hv.w = f32_to_bf16(gt[3] / (1.0f + expf(-gt[3])) * up[3]);
      *reinterpret_cast<ushort4 *>(hout + (size_t)row * ldy + o) = hv;
    }
  }
}

bool gemm_mfma_supported(int32_t n, int32_t K, int32_t O) {
  return n >= 1 && n <= TR_MAX_NODES && K % GEMM_KB == 0 && O % 16 == 0;
}

template <int NT>
static hipError_t launch_nt(const bf16_t *a, const bf16_t *w, const bf16_t *w2, int32_t n, int32_t K, int32_t O,
                            float *y, int32_t ldy, GemmMode mode, bf16_t *hout, hipStream_t st) {
  const dim3 grid(O / 16), block(GEMM_WAVES * 64);
  const size_t smem1 = (size_t)(GEMM_WAVES / 2) * NT * 64 * 16;
  switch (mode) {
  case GEMM_STORE:
    hipLaunchKernelGGL((k_gemm_mfma<NT, GEMM_STORE>), grid, block, smem1, st, a, w, w2, n, K, y, ldy, hout);
    break;
  case GEMM_ADD:
    hipLaunchKernelGGL((k_gemm_mfma<NT, GEMM_ADD>), grid, block, smem1, st, a, w, w2, n, K, y, ldy, hout);
    break;
  case GEMM_SWIGLU:
    hipLaunchKernelGGL((k_gemm_mfma<NT, GEMM_SWIGLU>), grid, block, 2 * smem1, st, a, w, w2, n, K, y, ldy, hout);
    break;
  }
  return hipGetLastError();
}

hipError_t launch_gemm_mfma(const bf16_t *a, const bf16_t *w, const bf16_t *w2, int32_t n, int32_t K, int32_t O,
                            float *y, int32_t ldy, GemmMode mode, bf16_t *hout, hipStream_t st) {
  switch ((n + 15) / 16) {
  case 1: return launch_nt<1>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  case 2: return launch_nt<2>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  case 3: return launch_nt<3>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  case 4: return launch_nt<4>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  case 5: return launch_nt<5>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  case 6: return launch_nt<6>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  case 7: return launch_nt<7>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  case 8: return launch_nt<8>(a, w, w2, n, K, O, y, ldy, mode, hout, st);
  }
  return hipErrorInvalidValue;
}

} // namespace tr
