// Tree attention on the matrix cores (Section 2.2 "Tree Attention"): head_dim 128, bf16 Q/K/V, float32
// softmax statistics and accumulators.  HBM-bound: every K/V byte of the head is read once per call.
//
// A workgroup owns HPW query heads that share one K/V head (HPW = 2 under grouped-query attention with an
// even group, else 1) and every nsplit-th 32-key tile; its waves own one (head, tile of 16 tree nodes)
// each, so no cross-wave reduction is needed.  K and V tiles are staged through LDS (double buffered,
// one barrier per tile) and shared by the waves, so two heads of a group read their K/V once instead of
// twice.  The grid is (K/V head, head group, split): workgroups that read the same K/V head have linear
// ids congruent modulo the number of K/V heads and, with 8 of those and round-robin dispatch, land on one
// XCD, whose L2 then serves the remaining re-reads.
//
// Everything is computed transposed so that no value ever changes lanes between the two contractions:
//   S^T[key][node] = K[key][:] . Q[node][:]      A = K tile (16 keys x 32 d), B = Q^T; lane l receives
//                                                keys 4*(l/16) .. +3 of node l%16
//   O^T[d][node]  += V^T[d][key] * P^T[key][node] A = V^T tile (16 d x 32 keys), B = P^T built in place from
//                                                the lane's own 8 probabilities (two 16-key S^T tiles)
// The KV cache is kept in exactly these operand orders (TR_KV_TILED, see kv_k_index / kv_v_index), so a
// tile is one contiguous 8 KiB block in memory and an LDS read of 16 bytes per lane is an MFMA operand.
//
// Mask: key position p is visible to node i when p < L (committed prefix), or L <= p < L + N and bit
// p - L of the node's ancestor mask is set.  Invisible keys get probability exactly 0.
// With more than one split, split s owns tiles s, s + nsplit, ...; each writes (max, sum, normalised O in
// half precision) per node and k_attn_merge combines them in split order.  K/V are read with streaming
// loads: they are used once per call and would otherwise push the activations out of L2.
#include "tr_kernels.h"

namespace tr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;

__device__ inline f32x4 mfma16a(const u32x4 &a, const u32x4 &b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

constexpr int ATT_TILE_BYTES = 16384; // 32 keys: K 8 KiB + V 8 KiB
constexpr float NEG_BIG = -1e30f;

template <int NT, int HPW>
__global__ __launch_bounds__(NT * HPW * 64) void k_attn_mfma(const bf16_t *__restrict__ q, const bf16_t *__restrict__ Kl,
                                                       const bf16_t *__restrict__ Vl, int32_t H, int32_t Hkv,
                                                       int32_t cap, int32_t n, const uint64_t *__restrict__ anc,
                                                       const int32_t *__restrict__ d_len, int32_t nsplit,
                                                       float *__restrict__ part_ml, float *__restrict__ part_acc,
                                                       bf16_t *__restrict__ out, int32_t out_row_tiles, int32_t row0) {
  constexpr int THREADS = NT * HPW * 64;
  constexpr int SLOTS = ATT_TILE_BYTES / 16;                 // 16-byte slots per tile
  constexpr int PER_THREAD = (SLOTS + THREADS - 1) / THREADS;
  // two tile buffers; reused at the end for one 4 KiB block per wave
  constexpr int LDS_SLOTS = 2 * SLOTS > NT * HPW * 256 ? 2 * SLOTS : NT * HPW * 256;
  __shared__ u32x4 lds_all[LDS_SLOTS];
  u32x4 (*lds)[SLOTS] = reinterpret_cast<u32x4 (*)[SLOTS]>(lds_all);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int wt = wave % NT;                                  // node tile of this wave
  // grid (K/V head, head group inside it, split): linear ids of one K/V head differ by multiples of Hkv
  const int hk = blockIdx.x, split = blockIdx.z;
  const int h = hk * (H / Hkv) + blockIdx.y * HPW + wave / NT;
  // split s owns tiles s, s + nsplit, s + 2 nsplit, ...: its first tile does not depend on the committed
  // length, so that fetch is issued before the length has arrived, and the masked tiles at the end of
  // the sequence spread over the splits

  const int node = wt * 16 + r;
  const int node_c = node < n ? node : n - 1;
  // Q^T operand: lane (node r, group g) holds Q[node][32c + 8g .. +7] for d-step c
  u32x4 qf[4];
  {
    const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + ((size_t)node_c * H + h) * 128 + 8 * g);
#pragma unroll
    for (int c = 0; c < 4; ++c) qf[c] = qp[c * 4];
  }
  const uint64_t a0 = anc[2 * node_c], a1 = anc[2 * node_c + 1];

  const u32x4 *Kh = reinterpret_cast<const u32x4 *>(Kl + (size_t)hk * cap * 128);
  const u32x4 *Vh = reinterpret_cast<const u32x4 *>(Vl + (size_t)hk * cap * 128);

  f32x4 acc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  // running sum l of the (bf16-rounded) probabilities, kept as the product of an all-ones A tile with
  // P^T: every row of that product is the column sum, so each lane ends with l of its own node
  f32x4 accl = f32x4{0.f, 0.f, 0.f, 0.f};
  const u32x4 ones = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  float m = NEG_BIG;
  const float sc = 0.08838834764831845f * 1.4426950408889634f; // 1/sqrt(128) * log2(e)

  // K/V tiles travel global -> registers -> LDS with one tile of loads in flight.  More were measured and
  // are no faster: with one query head per K/V head the workgroups together already pull K/V at the HBM
  // rate, with shared K/V heads the per-tile chain of dependent steps (stage, barrier, score
  // contraction, softmax, value contraction) is the limit.
  u32x4 stage[PER_THREAD];
  auto fetch = [&](int tile) {
    // K tile: 512 slots at Kh + tile*512; V tile: 512 slots at Vh + tile*512
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int s = tid + i * THREADS;
      if (s < SLOTS)
        stage[i] = __builtin_nontemporal_load(s < 512 ? Kh + (size_t)tile * 512 + s : Vh + (size_t)tile * 512 + (s - 512));
    }
  };
  auto publish = [&](int buf) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int s = tid + i * THREADS;
      if (s < SLOTS) lds[buf][s] = stage[i];
    }
  };

  // The loop is bound by the vector ALU work per score, not by the K/V stream, so that work is kept
  // minimal: tiles that lie wholly in the committed prefix skip the mask, the scale is folded into the
  // exponent with one fma, the accumulators are rescaled only when some lane's maximum moved, and the
  // bf16 rounding of the probabilities is the hardware's packed conversion.
  if ((split + 1) * 32 <= cap) fetch(split); // inside the cache allocation even if beyond the sequence
  const int L = *d_len + row0;
  const int total = L + n;
  const int n_tiles = (total + 31) >> 5;
  int buf = 0;
  for (int t = split; t < n_tiles; t += nsplit, buf ^= 1) {
    publish(buf);
    __syncthreads();
    if (t + nsplit < n_tiles) fetch(t + nsplit);
    const u32x4 *kt = lds[buf];
    const u32x4 *vt = lds[buf] + 512;

    f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      s0 = mfma16a(kt[c * 64 + lane], qf[c], s0);
      s1 = mfma16a(kt[(4 + c) * 64 + lane], qf[c], s1);
    }
    const bool in_prefix = t * 32 + 32 <= L; // uniform: every key of the tile is visible to every node
    float pr[8];
    if (in_prefix) {
      float mx = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])), fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m, mx * sc);
      if (__any(m_new > m)) {
        const float corr = __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          acc[dt][0] *= corr; acc[dt][1] *= corr; acc[dt][2] *= corr; acc[dt][3] *= corr;
        }
        accl[0] *= corr; accl[1] *= corr; accl[2] *= corr; accl[3] *= corr;
        m = m_new;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pr[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[e], sc, -m));
        pr[4 + e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[e], sc, -m));
      }
    } else {
      float x[8];
      bool vis[8];
      const int pbase = t * 32 + 4 * g;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int p = pbase + (e >> 2) * 16 + (e & 3);
        bool v = p < L;
        if (!v && p < total) {
          const int j = p - L;
          v = j < 64 ? ((a0 >> j) & 1ull) : ((a1 >> (j - 64)) & 1ull);
        }
        vis[e] = v;
        const float sv = (e < 4 ? s0[e & 3] : s1[e & 3]) * sc;
        x[e] = v ? sv : NEG_BIG;
      }
      float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m, mx);
      if (__any(m_new > m)) {
        const float corr = __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          acc[dt][0] *= corr; acc[dt][1] *= corr; acc[dt][2] *= corr; acc[dt][3] *= corr;
        }
        accl[0] *= corr; accl[1] *= corr; accl[2] *= corr; accl[3] *= corr;
        m = m_new;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) pr[e] = vis[e] ? __builtin_amdgcn_exp2f(x[e] - m) : 0.f;
    }
    // P^T operand: the lane's own 8 probabilities, rounded to bf16 (round to nearest even)
    u32x4 pf;
#pragma unroll
    for (int e = 0; e < 8; e += 2)
      pf[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pr[e], pr[e + 1]}, bf16x2));
    accl = mfma16a(ones, pf, accl);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = mfma16a(vt[dt * 64 + lane], pf, acc[dt]);
  }
  const float lsum = accl[0];

  if (nsplit == 1) {
    if (node >= n) return;
    const float inv = 1.0f / lsum;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      const int d = 16 * dt + 4 * g;
      ushort4 o;
      o.x = f32_to_bf16(acc[dt][0] * inv); o.y = f32_to_bf16(acc[dt][1] * inv);
      o.z = f32_to_bf16(acc[dt][2] * inv); o.w = f32_to_bf16(acc[dt][3] * inv);
      const size_t idx = out_row_tiles > 0 ? act_frag_index(node + row0, h * 128 + d, out_row_tiles)
                                           : ((size_t)node * H + h) * 128 + d;
      store_stream(out + idx, o);
    }
    return;
  }
  // a split's partial result is its own normalised output (a convex combination of V rows, so it fits
  // half precision with 2^-11 relative error, below the bf16 rounding of the merged output) plus (m, l).
  // The wave's 16 x 128 block is turned through LDS so that a node's 256 bytes leave as whole lines.
  const size_t prow = ((size_t)split * H + h) * NP + wt * 16;
  if (g == 0 && node < n) {
    part_ml[(prow + r) * 2] = m;
    part_ml[(prow + r) * 2 + 1] = lsum;
  }
  const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
  __syncthreads(); // every wave is done with the last K/V tile
  // row r keeps its 16-byte chunk c at slot c ^ r, so the 16 rows of one store hit distinct banks
  char *blk = reinterpret_cast<char *>(lds_all) + wave * 4096;
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) {
    // clamped to the half-precision range: a value-cache entry beyond +-65504 saturates instead of
    // turning into an infinity that the merge would spread over the row
    f32x4 o = acc[dt] * inv;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = fminf(fmaxf(o[e], -65504.0f), 65504.0f);
    *reinterpret_cast<f16x4 *>(blk + r * 256 + (((2 * dt + (g >> 1)) ^ r) << 4) + 8 * (g & 1)) =
        __builtin_convertvector(o, f16x4);
  }
  // the wave reads back only what it wrote itself; its LDS operations complete in order
  asm volatile("" ::: "memory");
  u32x4 *pa = reinterpret_cast<u32x4 *>(part_acc);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = i * 64 + lane, rr = c >> 4, cc = c & 15;
    const u32x4 v = *reinterpret_cast<const u32x4 *>(blk + rr * 256 + ((cc ^ rr) << 4));
    if (wt * 16 + rr < n) pa[(prow + rr) * 16 + cc] = v; // plain store: the merge pass finds these in L2
  }
}

// ---------------------------------------------------------------------------------------------
// One-launch form for short sequences: a workgroup owns one (query head, tile of 16 nodes) and its eight
// waves split the keys (wave w takes the 32-key tiles w, w+8, ...), each reading its K/V tiles from memory
// straight into matrix-core operand registers (the cache layout is that order; nothing is shared between the
// waves, so nothing is staged).  The waves' (max, sum, accumulator) meet in LDS and wave w finishes features
// 16w .. 16w+15 of all 16 nodes, so no partial result ever leaves the compute unit and no merge launch
// follows.  The node tiles of a head read the same K/V: their workgroups are numbered so that round-robin
// placement puts them on one XCD, whose L2 serves the repeats.  Every compute unit then pulls the whole
// sequence of its head, (L + N) * 512 bytes, which is why this form is only chosen for short sequences.
// ---------------------------------------------------------------------------------------------
constexpr int ATT1_WAVES = 8;
constexpr size_t ATT1_LDS_BYTES = (size_t)ATT1_WAVES * 8 * 64 * 16 + (size_t)ATT1_WAVES * 16 * 2 * 4;
template <int DUMMY>
__global__ __launch_bounds__(ATT1_WAVES * 64) void k_attn_tile(const bf16_t *__restrict__ q, const bf16_t *__restrict__ Kl,
                                                             const bf16_t *__restrict__ Vl, int32_t H, int32_t Hkv,
                                                             int32_t cap, int32_t n, int32_t NT,
                                                             const uint64_t *__restrict__ anc,
                                                             const int32_t *__restrict__ d_len, bf16_t *__restrict__ out,
                                                             int32_t out_row_tiles, int32_t row0) {
  extern __shared__ f32x4 att1_lds[]; // ATT1_LDS_BYTES
  f32x4 (*s_acc)[8][64] = reinterpret_cast<f32x4 (*)[8][64]>(att1_lds);                         // [waves][8][64], 64 KiB
  float (*s_ml)[16][2] = reinterpret_cast<float (*)[16][2]>(att1_lds + ATT1_WAVES * 8 * 64);    // [waves][16][2]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  // linear id -> (head, node tile): ids that differ by 8 share a head's XCD; x = id % 8 picks the head inside
  // a block of 8 heads, y = id / 8 runs over (node tile, head block)
  const int id = blockIdx.x, x8 = id & 7, y = id >> 3;
  const int wt = y % NT, h = (y / NT) * 8 + x8;
  if (h >= H) return; // uniform over the workgroup (H not a multiple of 8)
  const int hk = h / (H / Hkv);

  const int node = wt * 16 + r;
  const int node_c = node < n ? node : n - 1;
  u32x4 qf[4];
  {
    const u32x4 *qp = reinterpret_cast<const u32x4 *>(q + ((size_t)node_c * H + h) * 128 + 8 * g);
#pragma unroll
    for (int c = 0; c < 4; ++c) qf[c] = qp[c * 4];
  }
  const uint64_t a0 = anc[2 * node_c], a1 = anc[2 * node_c + 1];
  const u32x4 *Kh = reinterpret_cast<const u32x4 *>(Kl + (size_t)hk * cap * 128) + lane;
  const u32x4 *Vh = reinterpret_cast<const u32x4 *>(Vl + (size_t)hk * cap * 128) + lane;

  f32x4 acc[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 accl = f32x4{0.f, 0.f, 0.f, 0.f};
  const u32x4 ones = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
  float m = NEG_BIG;
  const float sc = 0.08838834764831845f * 1.4426950408889634f; // 1/sqrt(128) * log2(e)

  u32x4 kq[2][8], vq[2][8]; // two tiles of operands in registers: the one in use and the next
  auto fetch = [&](int buf, int tile) {
#pragma unroll
    for (int c = 0; c < 8; ++c) kq[buf][c] = __builtin_nontemporal_load(Kh + (size_t)tile * 512 + c * 64);
#pragma unroll
    for (int c = 0; c < 8; ++c) vq[buf][c] = __builtin_nontemporal_load(Vh + (size_t)tile * 512 + c * 64);
  };
  if ((wave + 1) * 32 <= cap) fetch(0, wave); // inside the allocation even if beyond the sequence
  const int L = *d_len + row0;
  const int total = L + n;
  const int n_tiles = (total + 31) >> 5;
  int i = 0;
  for (int t = wave; t < n_tiles; t += ATT1_WAVES, ++i) {
    const bool has_next = t + ATT1_WAVES < n_tiles;
    // the buffers alternate by compile-time index: two copies of the body
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if ((i & 1) != b) continue;
      if (has_next) fetch(b ^ 1, t + ATT1_WAVES);
      f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        s0 = mfma16a(kq[b][c], qf[c], s0);
        s1 = mfma16a(kq[b][4 + c], qf[c], s1);
      }
      float xs[8];
      bool vis[8];
      const bool in_prefix = t * 32 + 32 <= L; // uniform: every key of the tile is visible to every node
      const int pbase = t * 32 + 4 * g;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int p = pbase + (e >> 2) * 16 + (e & 3);
        bool v = in_prefix || p < L;
        if (!v && p < total) {
          const int j = p - L;
          v = j < 64 ? ((a0 >> j) & 1ull) : ((a1 >> (j - 64)) & 1ull);
        }
        vis[e] = v;
        const float sv = (e < 4 ? s0[e & 3] : s1[e & 3]) * sc;
        xs[e] = v ? sv : NEG_BIG;
      }
      float mx = fmaxf(fmaxf(fmaxf(xs[0], xs[1]), fmaxf(xs[2], xs[3])), fmaxf(fmaxf(xs[4], xs[5]), fmaxf(xs[6], xs[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m, mx);
      if (__any(m_new > m)) {
        const float corr = __builtin_amdgcn_exp2f(m - m_new);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          acc[dt][0] *= corr; acc[dt][1] *= corr; acc[dt][2] *= corr; acc[dt][3] *= corr;
        }
        accl[0] *= corr; accl[1] *= corr; accl[2] *= corr; accl[3] *= corr;
        m = m_new;
      }
      float pr[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pr[e] = vis[e] ? __builtin_amdgcn_exp2f(xs[e] - m) : 0.f;
      u32x4 pf;
#pragma unroll
      for (int e = 0; e < 8; e += 2)
        pf[e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pr[e], pr[e + 1]}, bf16x2));
      accl = mfma16a(ones, pf, accl);
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) acc[dt] = mfma16a(vq[b][dt], pf, acc[dt]);
    }
  }

  // meet in LDS: every wave leaves its accumulators (unnormalised), its running maximum and its sum
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) s_acc[wave][dt][lane] = acc[dt];
  if (g == 0) {
    s_ml[wave][r][0] = m;
    s_ml[wave][r][1] = accl[0];
  }
  __syncthreads();
  // wave w finishes features 16w .. 16w+15: out = sum_v acc_v 2^(m_v - M) / sum_v l_v 2^(m_v - M) in wave order
  float M = NEG_BIG;
#pragma unroll
  for (int v = 0; v < ATT1_WAVES; ++v)
    if (s_ml[v][r][1] > 0.f) M = fmaxf(M, s_ml[v][r][0]);
  float den = 0.f;
  f32x4 num = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int v = 0; v < ATT1_WAVES; ++v) {
    const float lv = s_ml[v][r][1];
    if (lv > 0.f) {
      const float w = __builtin_amdgcn_exp2f(s_ml[v][r][0] - M);
      den += w * lv;
      num += s_acc[v][wave][lane] * w;
    }
  }
  if (node >= n) return;
  const float inv = 1.0f / den;
  const int d = 16 * wave + 4 * g;
  ushort4 o;
  o.x = f32_to_bf16(num[0] * inv); o.y = f32_to_bf16(num[1] * inv);
  o.z = f32_to_bf16(num[2] * inv); o.w = f32_to_bf16(num[3] * inv);
  const size_t idx = out_row_tiles > 0 ? act_frag_index(node + row0, h * 128 + d, out_row_tiles) : ((size_t)node * H + h) * 128 + d;
  store_stream(out + idx, o);
}

// out[node, h, :] = sum_s w_s o_s / sum_s w_s with w_s = l_s 2^(m_s - max m), o_s the split's normalised
// output; splits without visible keys (l_s == 0) contribute nothing.  Block (8 nodes, head), 32 threads x
// 4 features per node; all loads of a thread are issued before any arithmetic.
__global__ __launch_bounds__(256) void k_attn_merge(const float *__restrict__ part_ml, const float *__restrict__ part_acc,
                                                    int32_t H, int32_t n, int32_t nsplit, bf16_t *__restrict__ out,
                                                    int32_t out_row_tiles, int32_t row0) {
  const int node = blockIdx.x * 8 + (threadIdx.x >> 5), h = blockIdx.y, d = (threadIdx.x & 31) * 4;
  if (node >= n) return;
  float2 ml[ATTN_MAX_SPLITS];
  f16x4 av[ATTN_MAX_SPLITS];
#pragma unroll
  for (int s = 0; s < ATTN_MAX_SPLITS; ++s) {
    if (s < nsplit) {
      const size_t row = ((size_t)s * H + h) * NP + node;
      ml[s] = *reinterpret_cast<const float2 *>(part_ml + row * 2);
      av[s] = reinterpret_cast<const f16x4 *>(part_acc)[row * 32 + (d >> 2)];
    }
  }
  float M = NEG_BIG;
#pragma unroll
  for (int s = 0; s < ATTN_MAX_SPLITS; ++s)
    if (s < nsplit && ml[s].y > 0.f) M = fmaxf(M, ml[s].x);
  float den = 0.f;
  float4 num = float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < ATTN_MAX_SPLITS; ++s) {
    if (s < nsplit && ml[s].y > 0.f) {
      const float w = exp2f(ml[s].x - M) * ml[s].y;
      den += w;
      num.x += w * (float)av[s][0]; num.y += w * (float)av[s][1];
      num.z += w * (float)av[s][2]; num.w += w * (float)av[s][3];
    }
  }
  const float inv = 1.0f / den;
  ushort4 o;
  o.x = f32_to_bf16(num.x * inv); o.y = f32_to_bf16(num.y * inv);
  o.z = f32_to_bf16(num.z * inv); o.w = f32_to_bf16(num.w * inv);
  const size_t idx = out_row_tiles > 0 ? act_frag_index(node + row0, h * 128 + d, out_row_tiles)
                                       : ((size_t)node * H + h) * 128 + d;
  store_stream(out + idx, o);
}

int attn_heads_per_wg(int32_t H, int32_t Hkv, int32_t n) {
  const int G = H / Hkv, NT = (n + 15) / 16;
  return (G % 2 == 0 && NT * 2 <= 12) ? 2 : 1; // up to 12 waves keep 3 per SIMD and the registers they need
}

// As many key-axis splits as keep the launch within one workgroup per CU (a second workgroup on a CU
// shares that CU's memory rate and doubles the critical path), at least two 32-key tiles per split.
int attn_choose_splits(int32_t head_groups, int32_t len_bound) {
  const int tiles = (len_bound + 31) / 32;
  int s = 256 / (head_groups > 0 ? head_groups : 1);
  if (s > tiles / 2) s = tiles / 2;
  if (s > ATTN_MAX_SPLITS) s = ATTN_MAX_SPLITS;
  return s < 1 ? 1 : s;
}

template <int NT, int HPW>
static hipError_t launch_attn_k(const bf16_t *q, const bf16_t *Kl, const bf16_t *Vl, int32_t H, int32_t Hkv, int32_t cap,
                                int32_t n, const uint64_t *anc, const int32_t *d_len, int32_t nsplit, float *part_ml,
                                float *part_acc, bf16_t *out, int32_t out_row_tiles, int32_t row0, KernelTimer tm, hipStream_t st) {
  return launch(k_attn_mfma<NT, HPW>, dim3(Hkv, H / Hkv / HPW, nsplit), dim3(NT * HPW * 64), 0, st, tm, q, Kl, Vl, H, Hkv,
                cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0);
}

template <int NT>
static hipError_t launch_attn_nt(int hpw, const bf16_t *q, const bf16_t *Kl, const bf16_t *Vl, int32_t H, int32_t Hkv,
                                 int32_t cap, int32_t n, const uint64_t *anc, const int32_t *d_len, int32_t nsplit,
                                 float *part_ml, float *part_acc, bf16_t *out, int32_t out_row_tiles, int32_t row0, KernelTimer tm,
                                 hipStream_t st) {
  if constexpr (NT <= 6) {
    if (hpw == 2)
      return launch_attn_k<NT, 2>(q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st);
  }
  if (hpw != 1) return hipErrorInvalidValue;
  return launch_attn_k<NT, 1>(q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st);
}

// The one-launch form pays when a compute unit can pull its head's whole sequence in less time than the
// split form spends on its second launch: up to about this many positions (prefix + nodes), and only when few
// query heads share a K/V head (each of them re-reads it).  Measured at 32 heads, 80 nodes (us per layer, one
// launch / split + merge): 7.8 / 11.0 at 256 positions, 10.3 / 12.5 at 512, 12.5 / 13.3 at 768, 14.5 / 14.2
// at 1024, 22.2 / 17.9 at 2048.
constexpr int ATT1_MAX_LEN = 832;
bool attn_one_launch(int32_t H, int32_t Hkv, int32_t len_bound) { return len_bound <= ATT1_MAX_LEN && H / Hkv <= 2; }

hipError_t launch_attn_mfma(const bf16_t *q, const bf16_t *Kl, const bf16_t *Vl, int32_t H, int32_t Hkv, int32_t cap,
                            int32_t n, const uint64_t *anc, const int32_t *d_len, int32_t len_bound, float *part_ml,
                            float *part_acc, bf16_t *out, int32_t out_row_tiles, int32_t row0, Profiler *prof, hipStream_t st) {
  if (Hkv < 1 || H % Hkv != 0) return hipErrorInvalidValue;
  const KernelTimer tm = prof_next(prof, PC_ATTN);
  if (attn_one_launch(H, Hkv, len_bound)) {
    const int NT = (n + 15) / 16;
    static bool once = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_tile<0>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)ATT1_LDS_BYTES) == hipSuccess;
    if (!once) return hipErrorInvalidValue;
    return launch(k_attn_tile<0>, dim3(((H + 7) / 8) * 8 * NT), dim3(ATT1_WAVES * 64), ATT1_LDS_BYTES, st, tm, q, Kl, Vl,
                  H, Hkv, cap, n, NT, anc, d_len, out, out_row_tiles, row0);
  }
  const int hpw = attn_heads_per_wg(H, Hkv, n);
  const int nsplit = attn_choose_splits(H / hpw, len_bound);
  hipError_t e = hipErrorInvalidValue;
  switch ((n + 15) / 16) {
  case 1: e = launch_attn_nt<1>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  case 2: e = launch_attn_nt<2>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  case 3: e = launch_attn_nt<3>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  case 4: e = launch_attn_nt<4>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  case 5: e = launch_attn_nt<5>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  case 6: e = launch_attn_nt<6>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  case 7: e = launch_attn_nt<7>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  case 8: e = launch_attn_nt<8>(hpw, q, Kl, Vl, H, Hkv, cap, n, anc, d_len, nsplit, part_ml, part_acc, out, out_row_tiles, row0, tm, st); break;
  }
  if (e != hipSuccess || nsplit == 1) return e;
  return launch(k_attn_merge, dim3((n + 7) / 8, H), dim3(256), 0, st, prof_next(prof, PC_ATTN_MERGE), part_ml, part_acc, H,
                n, nsplit, out, out_row_tiles, row0);
}

} // namespace tr
