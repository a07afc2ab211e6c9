// Launch interfaces of the bf16 MFMA kernels (gfx950).
#pragma once
#include "tr_internal.h"

namespace tr {

enum GemmMode { GEMM_STORE = 0, GEMM_ADD = 1, GEMM_SWIGLU = 2 };

// y[n, O] = a[n, K] * w[O, K]^T with bf16 operands and float32 accumulation.
//   GEMM_STORE : y[r*ldy + o]  = acc
//   GEMM_ADD   : y[r*ldy + o] += acc                       (residual add, one owner per element)
//   GEMM_SWIGLU: hout[r*ldy + o] = bf16(silu(acc_w) * acc_w2)   (two weight matrices, y unused)
// Rows of `a` are read up to index n-1 only.
bool gemm_mfma_supported(int32_t n, int32_t K, int32_t O);
hipError_t launch_gemm_mfma(const bf16_t *a, const bf16_t *w, const bf16_t *w2, int32_t n, int32_t K, int32_t O,
                            float *y, int32_t ldy, GemmMode mode, bf16_t *hout, hipStream_t st);

// Tree attention for head_dim 128, bf16 K/V/Q, split over the key axis with a merge pass.
// len_bound: host upper bound of L + n (sizes the split count only).
bool attn_mfma_supported(int32_t hd, int32_t n);
hipError_t launch_attn_mfma(const bf16_t *q, const bf16_t *Kl, const bf16_t *Vl, int32_t H, int32_t Hkv, int32_t cap,
                            int32_t n, const uint64_t *anc, const int32_t *d_len, int32_t len_bound, float *part_ml,
                            float *part_acc, bf16_t *out, hipStream_t st);

} // namespace tr
