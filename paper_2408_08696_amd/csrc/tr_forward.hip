// Verification forward: one pass of a Llama-style decoder over the N tree nodes (Section 2.2).
// This file holds the orchestration and the shape-generic kernels (any head_dim, f32 or bf16
// storage, plain ALU arithmetic).  The bf16 hot shapes are routed to the MFMA kernels in
// tr_gemm_mfma.hip / tr_attn_mfma.hip.
//
// Arithmetic contract of the bf16 path (both generic and MFMA kernels): the residual stream, the
// softmax statistics, all accumulators and the logits are float32; operands of every contraction
// (normalised activations, rotated Q/K, V, attention output, SwiGLU output) are rounded to bf16.
// In the packed path the RMS scale is applied after the contraction (it is a per-row scalar), i.e.
// the rounded operand is x * gain instead of x * gain * scale.
#include "tr_internal.h"
#include "tr_kernels.h"

namespace tr {

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static bool packed_supported(const tr_model &m);

Workspace plan_workspace(const tr_model &m) {
  Workspace w;
  const bool generic = !packed_supported(m); // the packed path keeps neither raw Q/K/V nor gate/up outputs
  const size_t esz = dtype_size(m.dtype);
  const size_t hq = (size_t)m.n_heads * m.head_dim, hk = (size_t)m.n_kv_heads * m.head_dim;
  const size_t R = generic ? NP : NPW; // rows of the activation buffers
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  w.x = take(R * m.d_model * 4);
  w.xn = take(R * m.d_model * esz);
  w.qkv = take(generic ? (size_t)NP * (hq + 2 * hk) * 4 : 0);
  w.q = take(R * hq * esz);
  w.attn = take(R * hq * esz);
  w.gu = take(generic ? (size_t)NP * 2 * m.d_ffn * 4 : 0);
  w.h = take(R * m.d_ffn * esz);
  w.rope = take(R * m.head_dim * 4);
  w.logits = take((size_t)NP * m.vocab * 4);
  w.part_ml = take((size_t)ATTN_MAX_SPLITS * NP * m.n_heads * 2 * 4);
  w.part_acc = take((size_t)ATTN_MAX_SPLITS * NP * m.n_heads * m.head_dim * 4);
  w.ypart = take((generic ? (size_t)GEMM_MAX_SPLITS * NP : (size_t)WIDE_MAX_SPLITS * NPW) * m.d_model * 4);
  static_assert(WIDE_MAX_SPLITS * NPW >= GEMM_MAX_SPLITS * NP, "ypart serves both paths");
  w.ssq = take(R * ((m.d_model + 1023) / 1024) * 4);
  w.total = off;
  return w;
}

// ---------------------------------------------------------------------------------------------
// Embedding gather + rotary table.  Row n: x[n,:] = E[tok[n],:]; cos/sin of (L + depth[n]) * f_i
// with f_i = theta^(-2i/hd), evaluated in double so that long positions keep float32 accuracy.
// depth == nullptr: row n sits n positions after L (a run of consecutive prompt tokens).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_embed_rope(const T *__restrict__ E, int32_t V, int32_t d,
                                                    const int32_t *__restrict__ tok, const int32_t *__restrict__ depth,
                                                    const int32_t *__restrict__ d_len, int32_t hd, float theta,
                                                    float *__restrict__ x, float *__restrict__ rope) {
  const int n = blockIdx.x;
  int t = tok[n];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  const T *src = E + (size_t)t * d;
  for (int j = threadIdx.x; j < d; j += blockDim.x) x[(size_t)n * d + j] = to_f32<T>(src[j]);
  const int half = hd / 2;
  const double pos = (double)(*d_len + (depth != nullptr ? depth[n] : n));
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double f = pow((double)theta, -2.0 * (double)i / (double)hd);
    double sn, cs;
    sincos(pos * f, &sn, &cs);
    rope[(size_t)n * hd + i] = (float)cs;
    rope[(size_t)n * hd + half + i] = (float)sn;
  }
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: out[n,:] = T(x[n,:] * rsqrt(mean(x^2) + eps) * g)
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const float *__restrict__ x, const T *__restrict__ g, int32_t d,
                                                 float eps, T *__restrict__ out) {
  __shared__ float red[4];
  const int n = blockIdx.x;
  const float *row = x + (size_t)n * d;
  float ss = 0.f;
  for (int j = threadIdx.x; j < d; j += 256) {
    const float v = row[j];
    ss += v * v;
  }
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (red[0] + red[1]) + (red[2] + red[3]);
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
  for (int j = threadIdx.x; j < d; j += 256) out[(size_t)n * d + j] = from_f32<T>(row[j] * r * to_f32<T>(g[j]));
}

// ---------------------------------------------------------------------------------------------
// Generic linear: y[n,o] (+)= sum_k a[n,k] * w[o,k].  One wave per output feature and group of 16
// rows; lanes stride over k.  mode 0 = store, 1 = accumulate into y (residual add).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_linear_generic(const T *__restrict__ a, const T *__restrict__ w, int32_t n,
                                                        int32_t K, int32_t O, float *__restrict__ y, int32_t ldy,
                                                        int32_t mode) {
  const int lane = threadIdx.x & 63;
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n0 = blockIdx.y * 16;
  if (o >= O) return;
  float acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.f;
  const T *wr = w + (size_t)o * K;
  for (int kk = lane; kk < K; kk += 64) {
    const float wv = to_f32<T>(wr[kk]);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int r = n0 + j;
      const float av = r < n ? to_f32<T>(a[(size_t)r * K + kk]) : 0.f;
      acc[j] += wv * av;
    }
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    float v = acc[j];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    acc[j] = v;
  }
  if (lane < 16 && n0 + lane < n) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (j == lane) v = acc[j];
    float *dst = y + (size_t)(n0 + lane) * ldy + o;
    *dst = mode ? (*dst + v) : v;
  }
}

template <typename T>
static hipError_t linear_generic(const void *a, const void *w, int32_t n, int32_t K, int32_t O, float *y, int32_t ldy,
                                 int32_t mode, hipStream_t st, KernelTimer tm = KernelTimer{}) {
  return launch(k_linear_generic<T>, dim3((O + 3) / 4, (n + 15) / 16), dim3(256), 0, st, tm, (const T *)a, (const T *)w, n,
                K, O, y, ldy, mode);
}

// h[n,f] = T(silu(g) * u) with gu = [gate | up], each F wide
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu(const float *__restrict__ gu, int32_t F, T *__restrict__ h) {
  const int n = blockIdx.y;
  const int f = blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const float g = gu[(size_t)n * 2 * F + f], u = gu[(size_t)n * 2 * F + F + f];
  h[(size_t)n * F + f] = from_f32<T>(g / (1.0f + expf(-g)) * u);
}

// ---------------------------------------------------------------------------------------------
// Rotary embedding + KV write.  Block (n, head) over the concatenated [q heads | k heads | v heads].
// Rotated q -> q[n, h, :]; rotated k -> K[layer][h][L+n][:]; v -> V[layer][h][:][L+n].
// ---------------------------------------------------------------------------------------------
constexpr int ROPE_HPB = 8; // heads per block
template <typename T>
__global__ __launch_bounds__(256) void k_rope_kv(const float *__restrict__ qkv, int32_t n_part, size_t part_stride,
                                                 const float *__restrict__ rope, int32_t H, int32_t Hkv, int32_t hd,
                                                 int32_t cap,
                                                 const int32_t *__restrict__ d_len, T *__restrict__ q,
                                                 T *__restrict__ Kl, T *__restrict__ Vl, int32_t tiled) {
  const int n = blockIdx.x;
  const int half = hd / 2;
  const int heads = H + 2 * Hkv;
  const int width = heads * hd;
  const int pos = *d_len + n;
  const float *row = qkv + (size_t)n * width;
  // work item = (head, i): elements i and i + hd/2 of that head (a rotation pair for q and k heads)
  const int items = ROPE_HPB * half;
  for (int it = threadIdx.x; it < items; it += 256) {
    const int hh = blockIdx.y * ROPE_HPB + it / half, i = it % half;
    if (hh >= heads) break;
    const float *src = row + (size_t)hh * hd;
    // the projection may arrive as n_part K-split partial sums, added here in split order
    float a = src[i], b = src[i + half];
    for (int s = 1; s < n_part; ++s) {
      a += src[(size_t)s * part_stride + i];
      b += src[(size_t)s * part_stride + i + half];
    }
    if (hh < H + Hkv) {
      const float c = rope[(size_t)n * hd + i], sn = rope[(size_t)n * hd + half + i];
      const float ra = a * c - b * sn, rb = b * c + a * sn;
      a = ra;
      b = rb;
    }
    const T ta = from_f32<T>(a), tb = from_f32<T>(b);
    if (hh < H) {
      T *dst = q + ((size_t)n * H + hh) * hd;
      dst[i] = ta;
      dst[i + half] = tb;
    } else if (hh < H + Hkv) {
      if (tiled) {
        T *dst = Kl + (size_t)(hh - H) * cap * hd;
        dst[kv_k_index(pos, i)] = ta;
        dst[kv_k_index(pos, i + half)] = tb;
      } else {
        T *dst = Kl + ((size_t)(hh - H) * cap + pos) * hd;
        dst[i] = ta;
        dst[i + half] = tb;
      }
    } else {
      T *dst = Vl + (size_t)(hh - H - Hkv) * hd * cap;
      if (tiled) {
        dst[kv_v_index(pos, i)] = ta;
        dst[kv_v_index(pos, i + half)] = tb;
      } else {
        dst[(size_t)i * cap + pos] = ta;
        dst[(size_t)(i + half) * cap + pos] = tb;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Generic tree attention (Section 2.2 "Tree Attention"): block (node n, head h).  Keys are the
// committed positions 0..L-1 and the tree nodes j whose bit is set in anc[n] (cache position L+j);
// everything else is skipped exactly.  Online softmax over chunks of 256 keys.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_attn_generic(const T *__restrict__ q, const T *__restrict__ Kl,
                                                      const T *__restrict__ Vl, int32_t H, int32_t Hkv, int32_t hd,
                                                      int32_t cap, int32_t n_nodes, const uint64_t *__restrict__ anc,
                                                      const int32_t *__restrict__ d_len, T *__restrict__ out,
                                                      int32_t out_row_tiles) {
  __shared__ float sq[256];
  __shared__ float sp[256];
  __shared__ float red[4];
  const int n = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int hk = h / (H / Hkv);
  const int L = *d_len;
  const uint64_t a0 = anc[2 * n], a1 = anc[2 * n + 1];
  const T *Kh = Kl + (size_t)hk * cap * hd;
  const T *Vh = Vl + (size_t)hk * hd * cap;
  if (tid < hd) sq[tid] = to_f32<T>(q[((size_t)n * H + h) * hd + tid]);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)hd);
  float m = -1e30f, l = 0.f, acc = 0.f; // acc: output element tid (< hd)
  const int total = L + n_nodes;
  for (int base = 0; base < total; base += 256) {
    const int j = base + tid;
    bool vis = j < L;
    if (!vis && j < total) {
      const int t = j - L;
      vis = t < 64 ? ((a0 >> t) & 1) : ((a1 >> (t - 64)) & 1);
    }
    float s = -1e30f;
    if (vis) {
      const T *kr = Kh + (size_t)j * hd;
      float dot = 0.f;
      for (int e = 0; e < hd; ++e) dot += sq[e] * to_f32<T>(kr[e]);
      s = dot * scale;
    }
    float cm = s;
    for (int off = 32; off > 0; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off));
    if ((tid & 63) == 0) red[tid >> 6] = cm;
    __syncthreads();
    cm = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float m_new = fmaxf(m, cm);
    const float p = vis ? expf(s - m_new) : 0.f;
    sp[tid] = p;
    float ps = p;
    for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
    __syncthreads(); // red (max) consumed by everyone, sp complete
    if ((tid & 63) == 0) red[tid >> 6] = ps;
    __syncthreads();
    const float corr = expf(m - m_new);
    l = l * corr + ((red[0] + red[1]) + (red[2] + red[3]));
    m = m_new;
    if (tid < hd) {
      acc *= corr;
      const T *vr = Vh + (size_t)tid * cap + base;
      const int cnt = total - base < 256 ? total - base : 256;
      for (int e = 0; e < cnt; ++e) {
        const float pe = sp[e];
        if (pe != 0.f) acc += pe * to_f32<T>(vr[e]);
      }
    }
    __syncthreads();
  }
  if (tid < hd) {
    // row-major [n, H*hd], or fragment order for the o-projection when out_row_tiles > 0
    const size_t idx = out_row_tiles > 0 ? act_frag_index(n, h * hd + tid, out_row_tiles)
                                         : ((size_t)n * H + h) * hd + tid;
    out[idx] = from_f32<T>(acc / l);
  }
}

// ---------------------------------------------------------------------------------------------
// orchestration
// ---------------------------------------------------------------------------------------------
#define TR_TRY(expr)                   \
  do {                                 \
    hipError_t e__ = (expr);           \
    if (e__ != hipSuccess) return e__; \
  } while (0)

template <typename T>
static hipError_t attention_dispatch(const tr_kv &kv, int32_t layer, int32_t H, const TreeDev &tree, int32_t n,
                                     const T *q, T *out, int32_t out_row_tiles, float *part_ml, float *part_acc,
                                     Profiler *prof, hipStream_t st) {
  const size_t lsz = (size_t)kv.n_kv_heads * kv.capacity * kv.head_dim;
  const T *Kl = (const T *)kv.k + (size_t)layer * lsz;
  const T *Vl = (const T *)kv.v + (size_t)layer * lsz;
  if (kv.layout == TR_KV_TILED) {
    return launch_attn_mfma((const bf16_t *)q, (const bf16_t *)Kl, (const bf16_t *)Vl, H, kv.n_kv_heads, kv.capacity,
                            n, tree.anc, kv.d_len, kv.len_bound + n, part_ml, part_acc, (bf16_t *)out, out_row_tiles,
                            0, prof, st);
  }
  return launch(k_attn_generic<T>, dim3(n, H), dim3(256), 0, st, prof_next(prof, PC_ATTN), q, Kl, Vl, H, kv.n_kv_heads,
                kv.head_dim, kv.capacity, n, tree.anc, kv.d_len, out, out_row_tiles);
}

// ---------------------------------------------------------------------------------------------
// generic forward: row-major weights, any shape, f32 or bf16 storage
// ---------------------------------------------------------------------------------------------
template <typename T>
static hipError_t forward_generic(const tr_model &m, const tr_kv &kv, const TreeDev &tree, int32_t n,
                                  const int32_t *tok, float *logits_out, unsigned char *ws, Profiler *prof,
                                  hipStream_t st) {
  const Workspace w = plan_workspace(m);
  const int d = m.d_model, H = m.n_heads, Hkv = m.n_kv_heads, hd = m.head_dim, F = m.d_ffn;
  const int hq = H * hd, hk = Hkv * hd, wq = hq + 2 * hk;
  float *x = (float *)(ws + w.x);
  T *xn = (T *)(ws + w.xn);
  float *qkv = (float *)(ws + w.qkv);
  T *q = (T *)(ws + w.q);
  T *attn = (T *)(ws + w.attn);
  float *gu = (float *)(ws + w.gu);
  T *hbuf = (T *)(ws + w.h);
  float *rope = (float *)(ws + w.rope);
  const size_t lsz = (size_t)Hkv * kv.capacity * hd;

  TR_TRY(launch(k_embed_rope<T>, dim3(n), dim3(256), 0, st, prof_next(prof, PC_EMBED), (const T *)m.embed, m.vocab, d, tok,
                tree.depth, kv.d_len, hd, m.rope_theta, x, rope));
  for (int l = 0; l < m.n_layers; ++l) {
    const tr_layer &lw = m.layers[l];
    TR_TRY(launch(k_rmsnorm<T>, dim3(n), dim3(256), 0, st, prof_next(prof, PC_NORM), x, (const T *)lw.attn_norm, d,
                  m.rms_eps, xn));
    TR_TRY(linear_generic<T>(xn, lw.wq, n, d, hq, qkv, wq, 0, st, prof_next(prof, PC_QKV)));
    TR_TRY(linear_generic<T>(xn, lw.wk, n, d, hk, qkv + hq, wq, 0, st, prof_next(prof, PC_QKV)));
    TR_TRY(linear_generic<T>(xn, lw.wv, n, d, hk, qkv + hq + hk, wq, 0, st, prof_next(prof, PC_QKV)));
    TR_TRY(launch(k_rope_kv<T>, dim3(n, (H + 2 * Hkv + ROPE_HPB - 1) / ROPE_HPB), dim3(256), 0, st,
                  prof_next(prof, PC_ROPE), qkv, 1, (size_t)0, rope, H, Hkv, hd, kv.capacity, kv.d_len, q,
                  (T *)kv.k + (size_t)l * lsz, (T *)kv.v + (size_t)l * lsz, kv.layout));
    TR_TRY(attention_dispatch<T>(kv, l, H, tree, n, q, attn, 0, (float *)(ws + w.part_ml), (float *)(ws + w.part_acc),
                                 prof, st));
    TR_TRY(linear_generic<T>(attn, lw.wo, n, hq, d, x, d, 1, st, prof_next(prof, PC_OPROJ)));
    TR_TRY(launch(k_rmsnorm<T>, dim3(n), dim3(256), 0, st, prof_next(prof, PC_NORM), x, (const T *)lw.ffn_norm, d,
                  m.rms_eps, xn));
    TR_TRY(linear_generic<T>(xn, lw.w_gate, n, d, F, gu, 2 * F, 0, st, prof_next(prof, PC_GATEUP)));
    TR_TRY(linear_generic<T>(xn, lw.w_up, n, d, F, gu + F, 2 * F, 0, st, prof_next(prof, PC_GATEUP)));
    TR_TRY(launch(k_swiglu<T>, dim3((F + 255) / 256, n), dim3(256), 0, st, prof_next(prof, PC_GATEUP), gu, F, hbuf));
    TR_TRY(linear_generic<T>(hbuf, lw.w_down, n, F, d, x, d, 1, st, prof_next(prof, PC_DOWN)));
  }
  if (logits_out != nullptr) {
    TR_TRY(launch(k_rmsnorm<T>, dim3(n), dim3(256), 0, st, prof_next(prof, PC_NORM), x, (const T *)m.final_norm, d,
                  m.rms_eps, xn));
    TR_TRY(linear_generic<T>(xn, m.lm_head, n, d, m.vocab, logits_out, m.vocab, 0, st, prof_next(prof, PC_LMHEAD)));
  }
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// packed bf16 forward: MFMA GEMMs on packed weights, activations handed from kernel to kernel in
// fragment order, projection outputs that feed the residual stream kept as per-split partial sums
// which the next normalisation kernel folds into x in a fixed order.
// ---------------------------------------------------------------------------------------------
// Residual update and normalisation input, block (row, chunk of 1024 columns), 128 threads x 8 columns:
//   x[row, c] += sum_s part[s][row, c]        (n_part may be 0)
//   xg_frag    = bf16(x * g)                   fragment order; rows n..16*row_tiles-1 are zeros
//   ssq[row, chunk] = sum over the chunk of x^2
// The RMS scale 1/sqrt(mean(x^2) + eps) is a per-row scalar, so the GEMM that consumes xg_frag applies
// it to its output rows (gemm row_ssq arguments) instead of this kernel needing a whole-row reduction.
constexpr int NORM_CHUNK = 1024;
static_assert(NORM_CHUNK == 128 * 8, "one block iteration covers 128 threads x 8 columns");
__global__ __launch_bounds__(128) void k_add_frag(float *__restrict__ x, const float *__restrict__ part,
                                                  int32_t n_part, size_t part_stride, const bf16_t *__restrict__ g,
                                                  int32_t n, int32_t d, int32_t row_tiles,
                                                  bf16_t *__restrict__ xg_frag, float *__restrict__ ssq,
                                                  int32_t n_chunks) {
  __shared__ float red[2];
  const int row = blockIdx.x, chunk = blockIdx.y;
  const int j = chunk * NORM_CHUNK + threadIdx.x * 8;
  const bool live = row < n && j < d;
  float ss = 0.f;
  uint4 pk = uint4{0u, 0u, 0u, 0u};
  if (live) {
    float *xr = x + (size_t)row * d + j;
    float4 a = *reinterpret_cast<const float4 *>(xr), b = *reinterpret_cast<const float4 *>(xr + 4);
    for (int s = 0; s < n_part; ++s) {
      const float *pr = part + (size_t)s * part_stride + (size_t)row * d + j;
      const float4 pa = *reinterpret_cast<const float4 *>(pr), pb = *reinterpret_cast<const float4 *>(pr + 4);
      a.x += pa.x; a.y += pa.y; a.z += pa.z; a.w += pa.w;
      b.x += pb.x; b.y += pb.y; b.z += pb.z; b.w += pb.w;
    }
    if (n_part > 0) {
      *reinterpret_cast<float4 *>(xr) = a;
      *reinterpret_cast<float4 *>(xr + 4) = b;
    }
    const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    const uint4 gv = *reinterpret_cast<const uint4 *>(g + j);
    const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float g0 = bf16_to_f32((bf16_t)(gw[e] & 0xFFFFu)), g1 = bf16_to_f32((bf16_t)(gw[e] >> 16));
      o[e] = (uint32_t)f32_to_bf16(v[2 * e] * g0) | ((uint32_t)f32_to_bf16(v[2 * e + 1] * g1) << 16);
      ss += v[2 * e] * v[2 * e] + v[2 * e + 1] * v[2 * e + 1];
    }
    pk = uint4{o[0], o[1], o[2], o[3]};
  }
  if (j < d) *reinterpret_cast<uint4 *>(xg_frag + act_frag_index(row, j, row_tiles)) = pk;
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0 && row < n) ssq[(size_t)row * n_chunks + chunk] = red[0] + red[1];
}

// row-major bf16 [n, K] -> fragment order (standalone linear op only)
__global__ __launch_bounds__(256) void k_rows_to_frag(const bf16_t *__restrict__ a, int32_t n, int32_t K,
                                                      int32_t row_tiles, bf16_t *__restrict__ frag) {
  const int row = blockIdx.x;
  for (int j = threadIdx.x * 8; j < K; j += 2048) {
    uint4 v = uint4{0u, 0u, 0u, 0u};
    if (row < n) v = *reinterpret_cast<const uint4 *>(a + (size_t)row * K + j);
    *reinterpret_cast<uint4 *>(frag + act_frag_index(row, j, row_tiles)) = v;
  }
}

__global__ __launch_bounds__(256) void k_sum_parts(const float *__restrict__ part, int32_t n_part, size_t part_stride,
                                                   size_t count, float *__restrict__ y) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float v = part[i];
  for (int s = 1; s < n_part; ++s) v += part[(size_t)s * part_stride + i];
  y[i] = v;
}

static bool packed_supported(const tr_model &m) {
  const int hq = m.n_heads * m.head_dim, hk = m.n_kv_heads * m.head_dim;
  return m.dtype == TR_BF16 && m.layout == TR_PACKED && m.d_model % 32 == 0 && m.d_model <= 8 * NORM_CHUNK && m.d_ffn % 32 == 0 && hq % 32 == 0 &&
         hk % 32 == 0 && m.vocab % 32 == 0;
}

static hipError_t forward_packed(const tr_model &m, const tr_kv &kv, const TreeDev &tree, int32_t n, const int32_t *tok,
                                 float *logits_out, unsigned char *ws, Profiler *prof, hipStream_t st) {
  typedef bf16_t T;
  const Workspace w = plan_workspace(m);
  const int d = m.d_model, H = m.n_heads, Hkv = m.n_kv_heads, hd = m.head_dim, F = m.d_ffn;
  const int hq = H * hd, hk = Hkv * hd;
  const int NT = (n + 15) / 16;
  float *x = (float *)(ws + w.x);
  T *xn = (T *)(ws + w.xn);
  T *q = (T *)(ws + w.q);
  T *attn = (T *)(ws + w.attn);
  T *hbuf = (T *)(ws + w.h);
  float *rope = (float *)(ws + w.rope);
  float *ypart = (float *)(ws + w.ypart);
  const size_t ystride = (size_t)NP * d;
  const size_t lsz = (size_t)Hkv * kv.capacity * hd;
  float *ssq = (float *)(ws + w.ssq);
  const int nch = (d + NORM_CHUNK - 1) / NORM_CHUNK;

  TR_TRY(launch(k_embed_rope<T>, dim3(n), dim3(256), 0, st, prof_next(prof, PC_EMBED), (const T *)m.embed, m.vocab, d, tok,
                tree.depth, kv.d_len, hd, m.rope_theta, x, rope));
  int pending = 0; // partial sums waiting in ypart
  auto add_norm = [&](const void *gain) {
    return launch(k_add_frag, dim3(NT * 16, nch), dim3(128), 0, st, prof_next(prof, PC_NORM), x, ypart, pending, ystride,
                  (const T *)gain, n, d, NT, xn, ssq, nch);
  };
  for (int l = 0; l < m.n_layers; ++l) {
    const tr_layer &lw = m.layers[l];
    TR_TRY(add_norm(lw.attn_norm));
    {
      GemmArgs g{};
      g.a_frag = xn; g.n = n; g.K = d;
      g.seg[0] = GemmSeg{(const T *)lw.wq, hq / 16};
      g.seg[1] = GemmSeg{(const T *)lw.wk, hk / 16};
      g.seg[2] = GemmSeg{(const T *)lw.wv, hk / 16};
      g.n_seg = 3; g.mode = GEMM_STORE;
      g.row_ssq = ssq; g.n_ssq = nch; g.norm_dim = d; g.eps = m.rms_eps;
      // RoPE and the query / cache writes happen in the projection's epilogue (one K-split: the epilogue
      // needs complete sums); wq and wk are packed with interleaved rows for that
      g.rope = GemmRope{q, (T *)kv.k + (size_t)l * lsz, (T *)kv.v + (size_t)l * lsz, rope, kv.d_len,
                        H, Hkv, hd, kv.capacity, kv.layout};
      gemm_plan(g, 1);
      TR_TRY(launch_gemm_mfma(g, st, prof_next(prof, PC_QKV)));
    }
    TR_TRY(attention_dispatch<T>(kv, l, H, tree, n, q, attn, NT, (float *)(ws + w.part_ml), (float *)(ws + w.part_acc),
                                 prof, st));
    {
      GemmArgs g{};
      g.a_frag = attn; g.n = n; g.K = hq;
      g.seg[0] = GemmSeg{(const T *)lw.wo, d / 16};
      g.n_seg = 1; g.y = ypart; g.ldy = d; g.split_stride = ystride; g.mode = GEMM_STORE;
      gemm_plan(g, GEMM_MAX_SPLITS);
      pending = g.splits;
      TR_TRY(launch_gemm_mfma(g, st, prof_next(prof, PC_OPROJ)));
    }
    TR_TRY(add_norm(lw.ffn_norm));
    {
      GemmArgs g{};
      g.a_frag = xn; g.n = n; g.K = d;
      g.seg[0] = GemmSeg{(const T *)lw.w_gate, F / 16};
      g.n_seg = 1; g.w2 = (const T *)lw.w_up; g.h_frag = hbuf; g.mode = GEMM_SWIGLU;
      g.row_ssq = ssq; g.n_ssq = nch; g.norm_dim = d; g.eps = m.rms_eps;
      gemm_plan(g, 1);
      TR_TRY(launch_gemm_mfma(g, st, prof_next(prof, PC_GATEUP)));
    }
    {
      GemmArgs g{};
      g.a_frag = hbuf; g.n = n; g.K = F;
      g.seg[0] = GemmSeg{(const T *)lw.w_down, d / 16};
      g.n_seg = 1; g.y = ypart; g.ldy = d; g.split_stride = ystride; g.mode = GEMM_STORE;
      gemm_plan(g, GEMM_MAX_SPLITS);
      pending = g.splits;
      TR_TRY(launch_gemm_mfma(g, st, prof_next(prof, PC_DOWN)));
    }
  }
  if (logits_out != nullptr) {
    TR_TRY(add_norm(m.final_norm));
    GemmArgs g{};
    g.a_frag = xn; g.n = n; g.K = d;
    g.seg[0] = GemmSeg{(const T *)m.lm_head, m.vocab / 16};
    g.n_seg = 1; g.y = logits_out; g.ldy = m.vocab; g.split_stride = 0; g.mode = GEMM_STORE;
    g.row_ssq = ssq; g.n_ssq = nch; g.norm_dim = d; g.eps = m.rms_eps;
    gemm_plan(g, 1);
    TR_TRY(launch_gemm_mfma(g, st, prof_next(prof, PC_LMHEAD)));
  }
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// Prompt ingestion on the packed path: up to NPW rows per pass.  The projections take all rows at once
// (tr_gemm_wide.hip: the layer's weights are read from memory once per pass instead of once per 128 rows);
// attention runs per block of 128 rows with the chain masks, each block seeing the committed length plus the
// rows before it as its prefix (their keys and values are in the cache by then: the Q/K/V projection of the
// whole pass precedes it).  Same arithmetic per row as forward_packed with one K-split.
// ---------------------------------------------------------------------------------------------
static hipError_t forward_wide(const tr_model &m, const tr_kv &kv, const TreeDev &chain, int32_t n, const int32_t *tok,
                               unsigned char *ws, hipStream_t st) {
  typedef bf16_t T;
  const Workspace w = plan_workspace(m);
  const int d = m.d_model, H = m.n_heads, Hkv = m.n_kv_heads, hd = m.head_dim, F = m.d_ffn;
  const int hq = H * hd, hk = Hkv * hd;
  const int RT = (n + 15) / 16;
  float *x = (float *)(ws + w.x);
  T *xn = (T *)(ws + w.xn);
  T *q = (T *)(ws + w.q);
  T *attn = (T *)(ws + w.attn);
  T *hbuf = (T *)(ws + w.h);
  float *rope = (float *)(ws + w.rope);
  float *ypart = (float *)(ws + w.ypart);
  const size_t lsz = (size_t)Hkv * kv.capacity * hd;
  float *ssq = (float *)(ws + w.ssq);
  const int nch = (d + NORM_CHUNK - 1) / NORM_CHUNK;
  const KernelTimer no_timer{};
  const size_t ystride = (size_t)NPW * d;

  TR_TRY(launch(k_embed_rope<T>, dim3(n), dim3(256), 0, st, no_timer, (const T *)m.embed, m.vocab, d, tok,
                (const int32_t *)nullptr, kv.d_len, hd, m.rope_theta, x, rope));
  int pending = 0;
  auto add_norm = [&](const void *gain) {
    return launch(k_add_frag, dim3(RT * 16, nch), dim3(128), 0, st, no_timer, x, ypart, pending, ystride,
                  (const T *)gain, n, d, RT, xn, ssq, nch);
  };
  for (int l = 0; l < m.n_layers; ++l) {
    const tr_layer &lw = m.layers[l];
    TR_TRY(add_norm(lw.attn_norm));
    {
      GemmArgs g{};
      g.a_frag = xn; g.n = n; g.K = d;
      g.seg[0] = GemmSeg{(const T *)lw.wq, hq / 16};
      g.seg[1] = GemmSeg{(const T *)lw.wk, hk / 16};
      g.seg[2] = GemmSeg{(const T *)lw.wv, hk / 16};
      g.n_seg = 3; g.mode = GEMM_STORE;
      g.row_ssq = ssq; g.n_ssq = nch; g.norm_dim = d; g.eps = m.rms_eps;
      g.rope = GemmRope{q, (T *)kv.k + (size_t)l * lsz, (T *)kv.v + (size_t)l * lsz, rope, kv.d_len,
                        H, Hkv, hd, kv.capacity, kv.layout};
      TR_TRY(launch_gemm_wide(g, 1, nullptr, st));
    }
    if (l == m.n_layers - 1) break; // ingestion only needs the cache: nothing reads the last layer's output
    for (int r0 = 0; r0 < n; r0 += NP) {
      const int nb = n - r0 < NP ? n - r0 : NP;
      TR_TRY(launch_attn_mfma(q + (size_t)r0 * hq, (const T *)kv.k + (size_t)l * lsz, (const T *)kv.v + (size_t)l * lsz, H,
                              Hkv, kv.capacity, nb, chain.anc, kv.d_len, kv.len_bound + r0 + nb,
                              (float *)(ws + w.part_ml), (float *)(ws + w.part_acc), attn, RT, r0, nullptr, st));
    }
    {
      GemmArgs g{};
      g.a_frag = attn; g.n = n; g.K = hq;
      g.seg[0] = GemmSeg{(const T *)lw.wo, d / 16};
      g.n_seg = 1; g.y = ypart; g.ldy = d; g.split_stride = ystride; g.mode = GEMM_STORE;
      TR_TRY(launch_gemm_wide(g, WIDE_MAX_SPLITS, &pending, st));
    }
    TR_TRY(add_norm(lw.ffn_norm));
    {
      GemmArgs g{};
      g.a_frag = xn; g.n = n; g.K = d;
      g.seg[0] = GemmSeg{(const T *)lw.w_gate, F / 16};
      g.n_seg = 1; g.w2 = (const T *)lw.w_up; g.h_frag = hbuf; g.mode = GEMM_SWIGLU;
      g.row_ssq = ssq; g.n_ssq = nch; g.norm_dim = d; g.eps = m.rms_eps;
      TR_TRY(launch_gemm_wide(g, 1, nullptr, st));
    }
    {
      GemmArgs g{};
      g.a_frag = hbuf; g.n = n; g.K = F;
      g.seg[0] = GemmSeg{(const T *)lw.w_down, d / 16};
      g.n_seg = 1; g.y = ypart; g.ldy = d; g.split_stride = ystride; g.mode = GEMM_STORE;
      TR_TRY(launch_gemm_wide(g, WIDE_MAX_SPLITS, &pending, st));
    }
  }
  return hipSuccess;
}

static bool wide_supported(const tr_model &m, const tr_kv &kv) {
  return packed_supported(m) && kv.layout == TR_KV_TILED && kv.dtype == TR_BF16 && m.head_dim == 128 &&
         m.d_model >= 64 && m.d_ffn >= 64;
}

int32_t prefill_rows(const tr_model &m, const tr_kv &kv) { return wide_supported(m, kv) ? NPW : NP; }

hipError_t run_prefill_pass(const tr_model &m, const tr_kv &kv, const TreeDev &chain, int32_t n, const int32_t *d_tokens,
                            void *ws, hipStream_t st) {
  if (n > NP && wide_supported(m, kv) && n <= NPW) return forward_wide(m, kv, chain, n, d_tokens, (unsigned char *)ws, st);
  if (n > NP) return hipErrorInvalidValue;
  return run_forward(m, kv, chain, n, d_tokens, nullptr, ws, nullptr, st);
}

hipError_t run_forward(const tr_model &m, const tr_kv &kv, const TreeDev &tree, int32_t n, const int32_t *d_tokens,
                       float *write_logits, void *ws, Profiler *prof, hipStream_t st) {
  if (packed_supported(m)) return forward_packed(m, kv, tree, n, d_tokens, write_logits, (unsigned char *)ws, prof, st);
  if (m.dtype == TR_BF16)
    return forward_generic<bf16_t>(m, kv, tree, n, d_tokens, write_logits, (unsigned char *)ws, prof, st);
  return forward_generic<float>(m, kv, tree, n, d_tokens, write_logits, (unsigned char *)ws, prof, st);
}

bool model_layout_ok(const tr_model &m) { return m.layout == TR_ROW_MAJOR || packed_supported(m); }

hipError_t run_tree_attention(const tr_kv &kv, int32_t layer, int32_t H, const TreeDev &tree, const void *d_q,
                              void *d_out, void *ws, hipStream_t st) {
  // standalone op: the split partials sit at the start of the caller's workspace
  float *ml = (float *)ws;
  float *acc = ws ? (float *)((unsigned char *)ws + align256((size_t)ATTN_MAX_SPLITS * NP * H * 2 * 4)) : nullptr;
  if (kv.dtype == TR_BF16)
    return attention_dispatch<bf16_t>(kv, layer, H, tree, tree.n_nodes, (const bf16_t *)d_q, (bf16_t *)d_out, 0, ml,
                                      acc, nullptr, st);
  return attention_dispatch<float>(kv, layer, H, tree, tree.n_nodes, (const float *)d_q, (float *)d_out, 0, nullptr,
                                   nullptr, nullptr, st);
}

size_t linear_workspace_bytes(int32_t n, int32_t in_f, int32_t out_f, int32_t splits) {
  const size_t nt = (size_t)(n + 15) / 16;
  return align256(nt * 16 * in_f * 2) + align256((size_t)splits * n * out_f * 4);
}

hipError_t run_linear(const void *x, const void *w, int32_t dtype, int32_t layout, int32_t n, int32_t in_f,
                      int32_t out_f, int32_t splits, float *y, void *ws, hipStream_t st) {
  if (layout == TR_PACKED) {
    const int NT = (n + 15) / 16;
    bf16_t *frag = (bf16_t *)ws;
    float *part = (float *)((unsigned char *)ws + align256((size_t)NT * 16 * in_f * 2));
    TR_TRY(launch(k_rows_to_frag, dim3(NT * 16), dim3(256), 0, st, KernelTimer{}, (const bf16_t *)x, n, in_f, NT, frag));
    GemmArgs g{};
    g.a_frag = frag; g.n = n; g.K = in_f;
    g.seg[0] = GemmSeg{(const bf16_t *)w, out_f / 16};
    g.n_seg = 1; g.y = splits > 1 ? part : y; g.ldy = out_f;
    g.split_stride = (size_t)n * out_f; g.mode = GEMM_STORE;
    if (n > NP) { // the prompt-ingestion kernel; it may use fewer splits than allowed
      TR_TRY(launch_gemm_wide(g, splits, &splits, st));
    } else {
      gemm_plan(g, splits);
      g.splits = splits; // the caller's split count is used as given
      TR_TRY(launch_gemm_mfma(g, st));
    }
    if (g.y != y) {
      const size_t count = (size_t)n * out_f;
      TR_TRY(launch(k_sum_parts, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, KernelTimer{}, part, splits,
                    (size_t)n * out_f, count, y));
    }
    return hipSuccess;
  }
  if (dtype == TR_BF16) return linear_generic<bf16_t>(x, w, n, in_f, out_f, y, out_f, 0, st);
  return linear_generic<float>(x, w, n, in_f, out_f, y, out_f, 0, st);
}

} // namespace tr
