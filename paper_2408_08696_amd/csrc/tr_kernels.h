// Launch interfaces of the bf16 MFMA kernels (gfx950).
#pragma once
#include "tr_internal.h"

namespace tr {

enum GemmMode { GEMM_STORE = 0, GEMM_SWIGLU = 2 };

// Streaming store for activations that the next kernel reads once: written through as issued, so the
// kernel does not end with dirty L2 lines to write back before its successor may start (the consumers
// mostly sit on other XCDs and read through memory anyway).  Measured per producer; it pays for the
// SwiGLU output and the attention output, not for K-split partial sums or the query / key writes.
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2s;
__device__ inline void store_stream(bf16_t *p, ushort4 v) {
  __builtin_nontemporal_store(u32x2s{(uint32_t)v.x | ((uint32_t)v.y << 16), (uint32_t)v.z | ((uint32_t)v.w << 16)},
                              reinterpret_cast<u32x2s *>(p));
}

// Fragment order (see tr_gemm_mfma.hip): a tile of 16 rows x 32 k is 64 lane slots of 8 bf16;
// element (row r, k) of an operand with T row tiles lives in tile (k/32, r/16) at lane slot
// (r%16) + 16*((k%32)/8), element k%8.  Weights use tile index (r/16) * (K/32) + k/32 instead.
__host__ __device__ inline size_t act_frag_index(int r, int k, int row_tiles) {
  return ((((size_t)(k >> 5) * row_tiles + (r >> 4)) * 64) + (r & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

struct GemmSeg {
  const bf16_t *w;   // packed weight matrix
  int32_t out_tiles; // its out_features / 16
};

// Optional epilogue of the fused Q/K/V projection (GEMM_STORE, splits == 1, q != nullptr): instead of
// storing y, rotate the query and key features (RoPE) and write queries, keys and values where the
// attention kernel reads them.  Needs wq and wk packed with their rows interleaved per head (feature i and
// i + head_dim/2 adjacent, see launch_pack_weight), so that a rotation pair sits in one lane; queries and
// cached keys then carry that feature order, which the attention dot product does not care about.
struct GemmRope {
  bf16_t *q;             // [n, H, hd] rotated queries; nullptr switches the epilogue off
  bf16_t *k_layer;       // this layer's K block of the cache
  bf16_t *v_layer;       // this layer's V block of the cache
  const float *rope;     // [rows, hd]: cos[hd/2] | sin[hd/2] of every row's position
  const int32_t *d_len;  // committed length L; row r is written at cache position L + r
  int32_t H, Hkv, hd, cap, tiled;
};

// y[n, O] = a[n, K] * W^T over the concatenation of up to three weight matrices (out-feature axis).
//   GEMM_STORE : y[split][row * ldy + o] = partial sum of that K-split (float32, row-major)
//   GEMM_SWIGLU: h_frag = bf16(silu(a W_gate^T) * (a W_up^T)) in fragment order over (k = o);
//                seg[0] = gate, w2 = up, splits must be 1
struct GemmArgs {
  const bf16_t *a_frag; // activations, fragment order, ceil(n/16) row tiles
  int32_t n, K;
  GemmSeg seg[3];
  int32_t n_seg;
  const bf16_t *w2;
  float *y;
  int32_t ldy;
  int32_t splits;
  size_t split_stride; // floats between consecutive partial results
  bf16_t *h_frag;
  int32_t mode;
  // optional RMS scale applied to output row r: 1/sqrt(sum_c row_ssq[r*n_ssq + c] / norm_dim + eps)
  const float *row_ssq;
  int32_t n_ssq, norm_dim;
  float eps;
  int32_t total_tiles;  // sum of seg[i].out_tiles
  int32_t tiles_per_wg; // most out-tiles (SWIGLU: gate/up tile pairs) a workgroup handles per pass
  int32_t groups;       // workgroups per K-split; each owns a contiguous ~total_tiles/groups out-tiles
  int32_t part_q, part_rem; // total_tiles / groups and total_tiles % groups (filled by launch_gemm_mfma)
  GemmRope rope;            // Q/K/V epilogue (see above), off when rope.q == nullptr
};

// Fills g.total_tiles, g.tiles_per_wg, g.groups and g.splits (<= max_splits; 1 for GEMM_SWIGLU).
void gemm_choose(int32_t n, int32_t K, int32_t total_tiles, bool swiglu, int32_t max_splits, int32_t *out_pmax,
                 int32_t *out_groups, int32_t *out_splits);
inline void gemm_plan(GemmArgs &g, int32_t max_splits) {
  int32_t total = 0;
  for (int i = 0; i < g.n_seg; ++i) total += g.seg[i].out_tiles;
  g.total_tiles = total;
  gemm_choose(g.n, g.K, total, g.mode == GEMM_SWIGLU, g.mode == GEMM_SWIGLU ? 1 : max_splits, &g.tiles_per_wg,
              &g.groups, &g.splits);
}

bool gemm_mfma_supported(int32_t n, int32_t K, int32_t O);
hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t st, KernelTimer tm = KernelTimer{});
// rope_hd > 0: packed row h*rope_hd + 2j + b takes source row h*rope_hd + j + b*rope_hd/2 (query / key
// matrices: the two features of a rotation pair become neighbours)
// Prompt ingestion: the same contraction and epilogues for up to WIDE_MAX_ROWS rows per launch (tr_gemm_wide.hip);
// a_frag / h_frag span ceil(n / 16) row tiles, rope rows are indexed by row; a plain store may be split over k
// into up to max_splits partial sums split_stride floats apart (*out_splits receives the count used).
constexpr int WIDE_MAX_ROWS = NPW;
constexpr int WIDE_MAX_SPLITS = 4;
bool gemm_wide_supported(int32_t n, int32_t K, int32_t O);
hipError_t launch_gemm_wide(const GemmArgs &g, int32_t max_splits, int32_t *out_splits, hipStream_t st,
                            KernelTimer tm = KernelTimer{});
hipError_t launch_pack_weight(const bf16_t *src, bf16_t *dst, int32_t O, int32_t K, int32_t rope_hd, hipStream_t st);

// Tree attention for head_dim 128, bf16 K/V/Q, split over the key axis with a merge pass.
// len_bound: host upper bound of L + n (sizes the split count only).
// Query heads one workgroup of launch_attn_mfma serves (they share a K/V head), and the key-axis splits it
// uses for H / that many head groups and this bound on committed length + nodes.
int attn_heads_per_wg(int32_t H, int32_t Hkv, int32_t n);
int attn_choose_splits(int32_t head_groups, int32_t len_bound);
// true: one launch without key splits or merge pass (short sequences); then the two values above do not apply
bool attn_one_launch(int32_t H, int32_t Hkv, int32_t len_bound);
// row0 (prompt ingestion in blocks of rows): the rows are rows row0 .. row0 + n - 1 of a longer pass whose
// keys and values are already cached; they see the committed length plus row0 positions as prefix, node j of
// this launch sits at that prefix length + j, and with out_row_tiles > 0 the output lands at row row0 + j.
hipError_t launch_attn_mfma(const bf16_t *q, const bf16_t *Kl, const bf16_t *Vl, int32_t H, int32_t Hkv, int32_t cap,
                            int32_t n, const uint64_t *anc, const int32_t *d_len, int32_t len_bound, float *part_ml,
                            float *part_acc, bf16_t *out, int32_t out_row_tiles, int32_t row0, Profiler *prof, hipStream_t st);

} // namespace tr
