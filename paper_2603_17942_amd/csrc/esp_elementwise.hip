// Glue kernels of the ESP decode step: block assembly, norms, rotary + KV append, SwiGLU,
// argmax, KV copies, mask-vector init / update.  All HBM-light; one pass over [rows, width].
#include <algorithm>

#include "esp_internal.h"

#define ESP_DISPATCH(dtype, ...)          \
  do {                                    \
    if ((dtype) == ESP_F32) {             \
      using T = float;                    \
      __VA_ARGS__;                        \
    } else {                              \
      using T = bf16_t;                   \
      __VA_ARGS__;                        \
    }                                     \
  } while (0)

__device__ __forceinline__ bool seq_ok(const KvDev& kv, int seq, int n_rows) {
  int L = kv.len[seq];
  int base = kv.base[seq];
  int cap = kv.seq_cap[seq];
  return L >= 0 && L <= kv.len_bound && n_rows >= 0 && L + n_rows <= cap && base >= 0 && (base & 63) == 0 &&
         (int64_t)base + cap <= kv.capacity;
}

__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return t;
}

// ---- block assembly (Sec. 3.1, Sec. 3.3): h0 rows and the per-row rotary table ---------------
template <typename T>
__global__ __launch_bounds__(256) void k_embed(BlockDev b, KvDev kv, const T* __restrict__ embed,
                                               const T* __restrict__ mask_embed, float* __restrict__ h, int d,
                                               int vocab, float* __restrict__ rope_tab, int hd, float theta,
                                               int32_t* status, size_t mask_seq_stride) {
  const int row = blockIdx.x;
  const int seq = row / b.rows_per_seq, r = row % b.rows_per_seq;
  const int nr = b.n_rows[seq];
  const bool ok = seq_ok(kv, seq, nr) && nr <= b.rows_per_seq;
  if (r == 0 && threadIdx.x == 0 && !ok) atomicOr(status, ESP_DEV_LEN_OVER_BOUND);
  const bool live = ok && r < nr;
  const T* src = nullptr;
  if (live) {
    int j = b.mask_j[row];
    if (j > 0) {
      if (j <= b.k_masks) src = mask_embed + seq * mask_seq_stride + (size_t)(j - 1) * d;
    } else {
      int t = b.tok[row];
      if (t < 0 || t >= vocab) {
        if (threadIdx.x == 0) atomicOr(status, ESP_DEV_BAD_TOKEN);
      } else {
        src = embed + (size_t)t * d;
      }
    }
  }
  float* hr = h + (size_t)row * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) hr[i] = src ? to_f32(src[i]) : 0.f;
  const int half = hd >> 1;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    // angle in double: positions reach 1e4..1e5 where an fp32 product loses the fraction
    double pos = live ? (double)(kv.len[seq] + b.depth[row]) : 0.0;
    double ang = pos * pow((double)theta, -2.0 * (double)i / (double)hd);
    rope_tab[((size_t)row * half + i) * 2 + 0] = (float)cos(ang);
    rope_tab[((size_t)row * half + i) * 2 + 1] = (float)sin(ang);
  }
}

hipError_t launch_embed(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, const void* embed,
                        const void* mask_embed, float* h, int d, int vocab, float* rope_tab, int hd,
                        float theta, int32_t* status, size_t mask_seq_stride) {
  int M = b.batch * b.rows_per_seq;
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_embed<T>, dim3(M), dim3(256), 0, st, b, kv, (const T*)embed,
                                         (const T*)mask_embed, h, d, vocab, rope_tab, hd, theta, status,
                                         mask_seq_stride));
  return hipGetLastError();
}

// ---- residual add of split-K partials + RMSNorm ------------------------------------------------
// One workgroup of 1024 threads per row; a thread owns float4 columns, so all split loads of a
// column are independent and in flight together.  d must be a multiple of 4.
template <typename T> struct Pack4;
template <> struct Pack4<float> {
  static __device__ __forceinline__ void store(float* p, f32x4_t v) { *reinterpret_cast<f32x4_t*>(p) = v; }
  static __device__ __forceinline__ f32x4_t load(const float* p) { return *reinterpret_cast<const f32x4_t*>(p); }
};
template <> struct Pack4<bf16_t> {
  static __device__ __forceinline__ void store(bf16_t* p, f32x4_t v) {
    bf16x4_t o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
    *reinterpret_cast<bf16x4_t*>(p) = o;
  }
  static __device__ __forceinline__ f32x4_t load(const bf16_t* p) {
    bf16x4_t i = *reinterpret_cast<const bf16x4_t*>(p);
    f32x4_t o = {(float)i[0], (float)i[1], (float)i[2], (float)i[3]};
    return o;
  }
};

template <typename T>
__global__ __launch_bounds__(1024) void k_residual_norm(float* __restrict__ h, const float* __restrict__ part,
                                                        int splits, size_t split_stride, int d,
                                                        const T* __restrict__ gain, float eps,
                                                        T* __restrict__ xn) {
  __shared__ float red[16];
  const size_t row = blockIdx.x;
  float* hr = h + row * d;
  const int d4 = d >> 2;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d4; i += 1024) {
    f32x4_t v = *reinterpret_cast<const f32x4_t*>(hr + 4 * i);
    for (int s = 0; s < splits; ++s)
      v += *reinterpret_cast<const f32x4_t*>(part + (size_t)s * split_stride + row * d + 4 * i);
    *reinterpret_cast<f32x4_t*>(hr + 4 * i) = v;
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += red[w];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = threadIdx.x; i < d4; i += 1024) {
    f32x4_t v = *reinterpret_cast<const f32x4_t*>(hr + 4 * i);   // written by this thread above
    f32x4_t g = Pack4<T>::load(gain + 4 * i);
    Pack4<T>::store(xn + row * d + 4 * i, v * inv * g);
  }
}

hipError_t launch_residual_norm(hipStream_t st, int dtype, float* h, const float* part, int splits, int M,
                                int d, const void* gain, float eps, void* xn_out) {
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_residual_norm<T>, dim3(M), dim3(1024), 0, st, h, part, splits,
                                         (size_t)M * d, d, (const T*)gain, eps, (T*)xn_out));
  return hipGetLastError();
}

// ---- QKV epilogue: split-K reduce, optional per-head RMSNorm, rotary, KV append ----------------
// one wave per (row, head); lane i < hd/2 owns the rotary pair (i, i + hd/2)
template <typename T>
__global__ __launch_bounds__(256) void k_qkv_post(BlockDev b, KvDev kv, int layer, const float* __restrict__ part,
                                                  int splits, size_t split_stride, int hq, int hkv, int hd,
                                                  int qk_norm, const T* __restrict__ qg, const T* __restrict__ kg,
                                                  float eps, const float* __restrict__ rope_tab,
                                                  T* __restrict__ q_out) {
  const int row = blockIdx.y;
  const int hidx = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int n_heads = hq + 2 * hkv;
  if (hidx >= n_heads) return;
  const int seq = row / b.rows_per_seq, r = row % b.rows_per_seq;
  const int nr = b.n_rows[seq];
  const bool live = seq_ok(kv, seq, nr) && nr <= b.rows_per_seq && r < nr;
  const int half = hd >> 1;
  const int ncol = n_heads * hd;
  const bool act = lane < half;
  float x0 = 0.f, x1 = 0.f;
  if (act && live) {
    size_t c0 = (size_t)row * ncol + (size_t)hidx * hd + lane;
    for (int s = 0; s < splits; ++s) {
      x0 += part[(size_t)s * split_stride + c0];
      x1 += part[(size_t)s * split_stride + c0 + half];
    }
  }
  if (hidx < hq + hkv) {
    if (qk_norm) {
      float ss = wave_sum(x0 * x0 + x1 * x1);
      float inv = 1.0f / sqrtf(ss / (float)hd + eps);
      const T* g = hidx < hq ? qg : kg;
      if (act) {
        x0 *= inv * to_f32(g[lane]);
        x1 *= inv * to_f32(g[lane + half]);
      }
    }
    if (!act) return;
    float c = rope_tab[((size_t)row * half + lane) * 2 + 0];
    float s = rope_tab[((size_t)row * half + lane) * 2 + 1];
    float y0 = x0 * c - x1 * s;
    float y1 = x1 * c + x0 * s;
    if (hidx < hq) {
      size_t o = ((size_t)row * hq + hidx) * hd + lane;
      q_out[o] = from_f32<T>(y0);
      q_out[o + half] = from_f32<T>(y1);
    } else if (live) {
      int kvh = hidx - hq;
      int64_t slot = (int64_t)kv.base[seq] + kv.len[seq] + r;
      T* kp = (T*)kv.k + kv_plane(layer, kvh, hkv, kv.capacity, hd);
      kp[k_off(slot, lane, hd)] = from_f32<T>(y0);
      kp[k_off(slot, lane + half, hd)] = from_f32<T>(y1);
    }
  } else if (act && live) {
    int kvh = hidx - hq - hkv;
    int64_t slot = (int64_t)kv.base[seq] + kv.len[seq] + r;
    T* vp = (T*)kv.v + kv_plane(layer, kvh, hkv, kv.capacity, hd);
    vp[v_off(slot, lane, hd)] = from_f32<T>(x0);
    vp[v_off(slot, lane + half, hd)] = from_f32<T>(x1);
  }
}

hipError_t launch_qkv_post(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int layer,
                           const float* part, int splits, int M, int hq, int hkv, int hd, int qk_norm,
                           const void* qg, const void* kg, float eps, const float* rope_tab, void* q_out) {
  int n_heads = hq + 2 * hkv;
  dim3 grid((n_heads + 3) / 4, M);
  size_t stride = (size_t)M * n_heads * hd;
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_qkv_post<T>, grid, dim3(256), 0, st, b, kv, layer, part, splits,
                                         stride, hq, hkv, hd, qk_norm, (const T*)qg, (const T*)kg, eps, rope_tab,
                                         (T*)q_out));
  return hipGetLastError();
}

// ---- SwiGLU over the fused gate/up GEMM output ---------------------------------------------------
// one thread per 4 consecutive features (d_ff multiple of 4)
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu(const float* __restrict__ part, int splits, size_t split_stride,
                                                int dff, T* __restrict__ act, size_t total4) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total4) return;
  const int per_row = dff >> 2;
  size_t row = i / per_row;
  int j = (int)(i % per_row) * 4;
  f32x4_t g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const float* p = part + (size_t)s * split_stride + row * 2 * dff;
    g += *reinterpret_cast<const f32x4_t*>(p + j);
    u += *reinterpret_cast<const f32x4_t*>(p + dff + j);
  }
  f32x4_t o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
  Pack4<T>::store(act + row * dff + j, o);
}

hipError_t launch_swiglu(hipStream_t st, int dtype, const float* part, int splits, int M, int dff, void* act) {
  size_t total4 = (size_t)M * (dff >> 2);
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_swiglu<T>, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, st,
                                         part, splits, (size_t)M * 2 * dff, dff, (T*)act, total4));
  return hipGetLastError();
}

// ---- argmax over the vocabulary, lowest id on ties ------------------------------------------------
__global__ __launch_bounds__(256) void k_argmax(const float* __restrict__ logits, size_t row_stride,
                                                const int32_t* __restrict__ row_map, int vocab,
                                                int32_t* __restrict__ out, const int32_t* __restrict__ out_index,
                                                const int32_t* __restrict__ draw_pos, uint32_t seed) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int m = blockIdx.x;
  const int dst = out_index ? out_index[m] : m;
  if (dst < 0) return;
  const size_t src = row_map ? (size_t)row_map[m] : (size_t)m;
  const float* p = logits + src * row_stride;
  const bool draw = draw_pos != nullptr;
  const uint32_t pos = draw ? (uint32_t)draw_pos[m] : 0u;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = threadIdx.x; i < vocab; i += 256) {
    float v = p[i];
    if (draw) v += gumbel_noise(seed, pos, (uint32_t)i);
    if (v > best) { best = v; bi = i; }   // ascending i per thread: first maximum is kept
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(best, o, 64);
    int oi = __shfl_xor(bi, o, 64);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
    out[dst] = bi == 0x7fffffff ? 0 : bi;
  }
}

hipError_t launch_argmax(hipStream_t st, const float* logits, size_t row_stride, const int32_t* row_map,
                         int n_rows_out, int vocab, int32_t* out, const int32_t* out_index,
                         const int32_t* draw_pos, uint32_t seed) {
  if (n_rows_out <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_argmax, dim3(n_rows_out), dim3(256), 0, st, logits, row_stride, row_map, vocab, out,
                     out_index, draw_pos, seed);
  return hipGetLastError();
}

// gather lists for the LM head over node rows: logical row m = seq*max_nodes + i
__global__ void k_node_rows(BlockDev b, int max_nodes, int32_t* a_rows, int32_t* out_rows,
                            const int32_t* __restrict__ kv_len, int32_t* pos_list) {
  int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m >= b.batch * max_nodes) return;
  int seq = m / max_nodes, i = m % max_nodes;
  int nn = b.n_nodes[seq];
  bool live = i < nn && nn <= b.n_rows[seq] && b.n_rows[seq] <= b.rows_per_seq;
  const int row = seq * b.rows_per_seq + (live ? i : 0);
  a_rows[m] = row;
  out_rows[m] = live ? seq * b.rows_per_seq + i : -1;
  if (pos_list) pos_list[m] = kv_len[seq] + b.depth[row] + 1;
}

hipError_t launch_node_rows(hipStream_t st, const BlockDev& b, int max_nodes, int32_t* a_rows,
                            int32_t* out_rows, const int32_t* kv_len, int32_t* pos_list) {
  int n = b.batch * max_nodes;
  hipLaunchKernelGGL(k_node_rows, dim3((n + 255) / 256), dim3(256), 0, st, b, max_nodes, a_rows, out_rows, kv_len,
                     pos_list);
  return hipGetLastError();
}

__global__ void k_row_positions(BlockDev b, const int32_t* __restrict__ kv_len, int32_t* pos_rows) {
  int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= b.batch * b.rows_per_seq) return;
  pos_rows[row] = kv_len[row / b.rows_per_seq] + b.depth[row] + 1;
}

hipError_t launch_row_positions(hipStream_t st, const BlockDev& b, const int32_t* kv_len, int32_t* pos_rows) {
  int n = b.batch * b.rows_per_seq;
  hipLaunchKernelGGL(k_row_positions, dim3((n + 255) / 256), dim3(256), 0, st, b, kv_len, pos_rows);
  return hipGetLastError();
}

// ---- plain rows <-> cache layout --------------------------------------------------------------------
template <typename T>
__global__ void k_kv_copy(KvDev kv, int layer, int n_kv, int hd, int seq_base, int first_slot, int n_slots,
                          T* k_rows, T* v_rows, int to_cache) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)n_slots * n_kv * hd;
  if (i >= total) return;
  int d = (int)(i % hd);
  int kvh = (int)((i / hd) % n_kv);
  int s = (int)(i / ((size_t)hd * n_kv));
  int64_t slot = (int64_t)seq_base + first_slot + s;
  T* kp = (T*)kv.k + kv_plane(layer, kvh, n_kv, kv.capacity, hd);
  T* vp = (T*)kv.v + kv_plane(layer, kvh, n_kv, kv.capacity, hd);
  if (to_cache) {
    kp[k_off(slot, d, hd)] = k_rows[i];
    vp[v_off(slot, d, hd)] = v_rows[i];
  } else {
    k_rows[i] = kp[k_off(slot, d, hd)];
    v_rows[i] = vp[v_off(slot, d, hd)];
  }
}

hipError_t launch_kv_copy(hipStream_t st, int dtype, const KvDev& kv, int layer, int n_kv, int hd, int seq_base,
                          int first_slot, int n_slots, void* k_rows, void* v_rows, int to_cache) {
  size_t total = (size_t)n_slots * n_kv * hd;
  if (total == 0) return hipSuccess;
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_kv_copy<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                                         kv, layer, n_kv, hd, seq_base, first_slot, n_slots, (T*)k_rows,
                                         (T*)v_rows, to_cache));
  return hipGetLastError();
}

// ---- mask vectors (Sec. 3.1 Eq. 4 and Eq. 5) -----------------------------------------------------------
template <typename T>
__global__ void k_mask_mean(const T* __restrict__ embed, const int32_t* __restrict__ tokens, int n, int k, int d,
                            int vocab, T* __restrict__ mask_embed) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d) return;
  float acc = 0.f;
  for (int t = 0; t < n; ++t) {
    int id = tokens[t];
    if (id >= 0 && id < vocab) acc += to_f32(embed[(size_t)id * d + i]);
  }
  T v = from_f32<T>(acc / (float)n);
  for (int j = 0; j < k; ++j) mask_embed[(size_t)j * d + i] = v;
}

hipError_t launch_mask_mean(hipStream_t st, int dtype, const void* embed, const int32_t* tokens, int n, int k,
                            int d, int vocab, void* mask_embed) {
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_mask_mean<T>, dim3((d + 255) / 256), dim3(256), 0, st, (const T*)embed,
                                         tokens, n, k, d, vocab, (T*)mask_embed));
  return hipGetLastError();
}

// Hard initialisation (Sec. 4, mask-design variant a): mask i = embedding of the prompt token
// k - i places before the end.
template <typename T>
__global__ void k_mask_last_k(const T* __restrict__ embed, const int32_t* __restrict__ tokens, int n, int k, int d,
                              int vocab, T* __restrict__ mask_embed) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d) return;
  for (int j = 0; j < k; ++j) {
    int id = tokens[n - k + j];
    mask_embed[(size_t)j * d + i] = id >= 0 && id < vocab ? embed[(size_t)id * d + i] : from_f32<T>(0.f);
  }
}

hipError_t launch_mask_last_k(hipStream_t st, int dtype, const void* embed, const int32_t* tokens, int n, int k,
                              int d, int vocab, void* mask_embed) {
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_mask_last_k<T>, dim3((d + 255) / 256), dim3(256), 0, st, (const T*)embed,
                                         tokens, n, k, d, vocab, (T*)mask_embed));
  return hipGetLastError();
}

// Gaussian fit to the embedding table (Sec. 4, variant b): mu[i] = mean over the vocabulary of
// column i, sigma = root mean square deviation of all entries from their column's mean.  Two
// passes over the table (mean, then squared deviations), each split into slabs of rows whose
// fp32 partial sums are added up in fp64, in slab order.
// MODE 0: partial[slab][i] = sum of column i over the slab; 1: sum of (x - mu[i])^2
template <typename T, int MODE>
__global__ __launch_bounds__(256) void k_embed_stats_partial(const T* __restrict__ embed, int vocab, int d,
                                                             int rows_per_slab, const float* __restrict__ mu,
                                                             float* __restrict__ partial) {
  const int i = blockIdx.x * 256 + threadIdx.x, slab = blockIdx.y;
  if (i >= d) return;
  const int v0 = slab * rows_per_slab, v1 = min(vocab, v0 + rows_per_slab);
  const float c = MODE ? mu[i] : 0.f;
  float acc = 0.f;
  for (int v = v0; v < v1; ++v) {
    const float x = to_f32(embed[(size_t)v * d + i]) - c;
    acc += MODE ? x * x : x;
  }
  partial[(size_t)slab * d + i] = acc;
}

__global__ __launch_bounds__(256) void k_embed_mean_final(const float* __restrict__ partial, int slabs, int d, int vocab,
                                                          float* __restrict__ mu) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= d) return;
  double s = 0.0;
  for (int b = 0; b < slabs; ++b) s += (double)partial[(size_t)b * d + i];
  mu[i] = (float)(s / (double)vocab);
}

// one workgroup: sigma = sqrt(sum of all partials / (vocab * d))
__global__ __launch_bounds__(256) void k_embed_sigma_final(const float* __restrict__ partial, int slabs, int d, int vocab,
                                                           float* __restrict__ sigma) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < d; i += 256)
    for (int b = 0; b < slabs; ++b) s += (double)partial[(size_t)b * d + i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) sigma[0] = (float)sqrt(red[0] / ((double)vocab * (double)d));
}

// m_j = mu + (shift + z_j) sigma; z: [k][d] standard normal draws of the caller, or null
template <typename T>
__global__ void k_mask_affine(const float* __restrict__ mu, const float* __restrict__ sigma,
                              const float* __restrict__ z, float shift, int k, int d, T* __restrict__ mask_embed) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d) return;
  const float sg = sigma[0], m = mu[i];
  for (int j = 0; j < k; ++j)
    mask_embed[(size_t)j * d + i] = from_f32<T>(fmaf(shift + (z ? z[(size_t)j * d + i] : 0.f), sg, m));
}

size_t mask_gaussian_scratch_floats(int d) { return (size_t)2 * d + 64; }   // least: one slab

hipError_t launch_mask_gaussian(hipStream_t st, int dtype, const void* embed, int vocab, int d, const float* z,
                                float shift, int k, float* scratch, size_t scratch_floats, void* mask_embed) {
  // scratch: mu [d], sigma [64 (one used)], partial [slabs][d]
  float* mu = scratch;
  float* sigma = scratch + d;
  float* partial = scratch + d + 64;
  const size_t room = (scratch_floats - d - 64) / d;
  const int slabs = (int)std::max<size_t>(1, std::min<size_t>(room, 256));
  const int rows_per_slab = (vocab + slabs - 1) / slabs;
  const int used = (vocab + rows_per_slab - 1) / rows_per_slab;
  const dim3 grid((d + 255) / 256, used);
  ESP_DISPATCH(dtype, hipLaunchKernelGGL((k_embed_stats_partial<T, 0>), grid, dim3(256), 0, st, (const T*)embed, vocab,
                                         d, rows_per_slab, (const float*)nullptr, partial));
  hipLaunchKernelGGL(k_embed_mean_final, dim3((d + 255) / 256), dim3(256), 0, st, partial, used, d, vocab, mu);
  ESP_DISPATCH(dtype, hipLaunchKernelGGL((k_embed_stats_partial<T, 1>), grid, dim3(256), 0, st, (const T*)embed, vocab,
                                         d, rows_per_slab, (const float*)mu, partial));
  hipLaunchKernelGGL(k_embed_sigma_final, dim3(1), dim3(256), 0, st, partial, used, d, vocab, sigma);
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_mask_affine<T>, dim3((d + 255) / 256), dim3(256), 0, st, mu, sigma, z, shift,
                                         k, d, (T*)mask_embed));
  return hipGetLastError();
}

template <typename T>
__global__ void k_mask_ema(const T* __restrict__ embed, const int32_t* __restrict__ n_emit,
                           const int32_t* __restrict__ emit_tok, float lambda, int k, int d, int vocab,
                           T* __restrict__ mask_embed) {
  // blockIdx.y: the sequence whose vectors ([k, d] at mask_embed + y * k * d) follow its own last
  // emitted token; a launch with one row of workgroups updates the shared vectors from sequence 0
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d) return;
  const int seq = blockIdx.y;
  int ne = n_emit[seq];
  if (ne < 1 || ne > ESP_MAX_MASKS + 1) return;
  int id = emit_tok[(size_t)seq * (ESP_MAX_MASKS + 1) + ne - 1];
  if (id < 0 || id >= vocab) return;
  float e = to_f32(embed[(size_t)id * d + i]);
  T* me = mask_embed + (size_t)seq * k * d;
  for (int j = 0; j < k; ++j) {
    float m = to_f32(me[(size_t)j * d + i]);
    me[(size_t)j * d + i] = from_f32<T>(m + lambda * (e - m));
  }
}

hipError_t launch_mask_ema(hipStream_t st, int dtype, const void* embed, const int32_t* n_emit,
                           const int32_t* emit_tok, float lambda, int k, int d, int vocab, void* mask_embed,
                           int n_seq) {
  ESP_DISPATCH(dtype, hipLaunchKernelGGL(k_mask_ema<T>, dim3((d + 255) / 256, n_seq), dim3(256), 0, st, (const T*)embed,
                                         n_emit, emit_tok, lambda, k, d, vocab, (T*)mask_embed));
  return hipGetLastError();
}
