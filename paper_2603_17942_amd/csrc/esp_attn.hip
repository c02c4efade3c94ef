// Tree-masked grouped-query attention of one decoder layer (paper Sec. 3.3, App. C, App. E).
//
// Row r of sequence b attends to cache slots [0, len[b]) and to the block rows c whose bit is set
// in its ancestor bitset (held at slots len[b] + c).  Only the last n_rows keys of a sequence need
// a mask test; every tile that lies inside the committed cache runs unmasked.
//
// bf16 / head_dim 128 path (k_attn_mfma): the G = n_q/n_kv query heads of a kv head times the
// block rows form the "query columns" of a (keys x queries) problem.  A workgroup owns W*32 query
// columns (W waves) and one split of the key range; K tiles ([64 keys][128]) and V tiles (already
// slot-contiguous per feature in HBM, [128][64]) are staged through LDS with register
// double-buffering and shared by the W waves.  S^T = K Q^T and O^T = V^T P^T both run on
// v_mfma_f32_32x32x16_bf16: computing the transposed scores leaves each lane with one query
// column and 16 keys per 32-key block, which is exactly the B-operand layout P^T needs, so the
// probabilities never leave registers.  Online softmax in fp32 (base-2 exponent), one exchange
// between the two lane halves per tile.  Partial (m, l, O) per split are merged by k_attn_merge in
// split order (fixed, so results do not depend on scheduling).
//
// Generic path (k_attn_generic): one wave per (row, head, split), any dtype / head_dim multiple of
// 64; used by the fp32 tiny configuration.
#include <algorithm>

#include "esp_internal.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float NEG_BIG = -1.0e30f;

__device__ __forceinline__ bool seq_ok(const KvDev& kv, int seq, int n_rows, int rows_per_seq) {
  int L = kv.len[seq];
  int base = kv.base[seq];
  int cap = kv.seq_cap[seq];
  return L >= 0 && L <= kv.len_bound && n_rows >= 0 && n_rows <= rows_per_seq && L + n_rows <= cap &&
         base >= 0 && (base & 63) == 0 && (int64_t)base + cap <= kv.capacity;
}

// --------------------------------------------------------------------------------------------------
template <typename T, int HD>
__global__ __launch_bounds__(64) void k_attn_generic(BlockDev b, KvDev kv, int layer, int hq, int hkv,
                                                     const T* __restrict__ q, float* __restrict__ part_o,
                                                     float* __restrict__ part_ml, int nsplit, int tps) {
  __shared__ float qs[HD];
  __shared__ float ps[64];
  const int row = blockIdx.x, h = blockIdx.y, sp = blockIdx.z, lane = threadIdx.x;
  const int seq = row / b.rows_per_seq, r = row % b.rows_per_seq;
  const int nr = b.n_rows[seq];
  if (!seq_ok(kv, seq, nr, b.rows_per_seq) || r >= nr) return;
  const int L = kv.len[seq], total = L + nr;
  const int ntiles = (total + 63) >> 6;
  const int t0 = sp * tps, t1 = min(ntiles, t0 + tps);
  const int kvh = h / (hq / hkv);
  const T* kp = (const T*)kv.k + kv_plane(layer, kvh, hkv, kv.capacity, HD);
  const T* vp = (const T*)kv.v + kv_plane(layer, kvh, hkv, kv.capacity, HD);
  const int64_t base = kv.base[seq];
  const float scale = LOG2E / sqrtf((float)HD);
  for (int d = lane; d < HD; d += 64) qs[d] = to_f32(q[((size_t)row * hq + h) * HD + d]) * scale;
  __syncthreads();
  const uint64_t* anc = b.anc + (size_t)row * b.anc_words;
  float m = NEG_BIG, l = 0.f;
  float o[HD / 64];
#pragma unroll
  for (int i = 0; i < HD / 64; ++i) o[i] = 0.f;
  for (int t = t0; t < t1; ++t) {
    const int key = t * 64 + lane;
    bool valid = key < total;
    if (valid && key >= L) {
      int c = key - L;
      valid = (anc[c >> 6] >> (c & 63)) & 1ull;
    }
    float s = NEG_BIG;
    if (valid) {
      const T* kr = kp + k_off(base + key, 0, HD);
      float acc = 0.f;
      for (int d = 0; d < HD; ++d) acc = fmaf(to_f32(kr[d]), qs[d], acc);
      s = acc;
    }
    float m_new = fmaxf(m, wave_max(s));
    float p = valid ? exp2f(s - m_new) : 0.f;
    float alpha = exp2f(m - m_new);
    l = l * alpha + wave_sum(p);
    m = m_new;
    ps[lane] = p;
    __syncthreads();
    const int nk = min(64, total - t * 64);
#pragma unroll
    for (int i = 0; i < HD / 64; ++i) {
      float a = o[i] * alpha;
      const T* vr = vp + v_off(base + t * 64, lane + 64 * i, HD);
      for (int kk = 0; kk < nk; ++kk) a = fmaf(ps[kk], to_f32(vr[kk]), a);
      o[i] = a;
    }
    __syncthreads();
  }
  const size_t item = ((size_t)row * hq + h) * nsplit + sp;
#pragma unroll
  for (int i = 0; i < HD / 64; ++i) part_o[item * HD + lane + 64 * i] = o[i];
  if (lane == 0) {
    part_ml[item * 2 + 0] = m;
    part_ml[item * 2 + 1] = l;
  }
}

// --------------------------------------------------------------------------------------------------
constexpr int K_ROW = 272;   // LDS bytes per key row: 256 + 16 (ds_read_b128 conflict-free over 8 rows)
constexpr int V_ROW = 136;   // LDS bytes per feature row: 128 + 8 (ds_read_b64 conflict-free over 16 rows)
constexpr int K_TILE_BYTES = 64 * K_ROW;
constexpr int V_TILE_BYTES = 128 * V_ROW;

// Tile staging.  Loads are unconditional (a piece index past the tile is clamped and its value
// dropped at the store) so that the staging registers stay in VGPRs.
template <int W>
__device__ __forceinline__ void attn_load_tile(const bf16_t* __restrict__ kt, const bf16_t* __restrict__ vt, int tid,
                                               uint4 (&kreg)[(1024 + 64 * W - 1) / (64 * W)],
                                               uint4 (&vreg)[(1024 + 64 * W - 1) / (64 * W)]) {
  constexpr int NT = 64 * W, PIECES = (1024 + NT - 1) / NT;
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    int p = min(tid + NT * i, 1023);
    kreg[i] = *reinterpret_cast<const uint4*>(kt + (size_t)p * 8);
    vreg[i] = *reinterpret_cast<const uint4*>(vt + (size_t)p * 8);
  }
}

// keys_left: keys of the tile that belong to the sequence; V of the others is zeroed (their
// probability is zero, but 0 * NaN from never-written cache memory would poison the MFMA)
template <int W>
__device__ __forceinline__ void attn_store_tile(unsigned char* ks, unsigned char* vs, int tid, int keys_left,
                                                const uint4 (&kreg)[(1024 + 64 * W - 1) / (64 * W)],
                                                const uint4 (&vreg)[(1024 + 64 * W - 1) / (64 * W)]) {
  constexpr int NT = 64 * W, PIECES = (1024 + NT - 1) / NT;
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    int p = tid + NT * i;
    if (p < 1024) {
      *reinterpret_cast<uint4*>(ks + (p >> 4) * K_ROW + (p & 15) * 16) = kreg[i];
      uint4 v = vreg[i];
      const int nv = keys_left - (p & 7) * 8;   // valid keys among the 8 of this piece
      // word w holds keys 2w (low half) and 2w+1 (high half)
      v.x &= nv >= 2 ? 0xffffffffu : (nv == 1 ? 0x0000ffffu : 0u);
      v.y &= nv >= 4 ? 0xffffffffu : (nv == 3 ? 0x0000ffffu : 0u);
      v.z &= nv >= 6 ? 0xffffffffu : (nv == 5 ? 0x0000ffffu : 0u);
      v.w &= nv >= 8 ? 0xffffffffu : (nv == 7 ? 0x0000ffffu : 0u);
      unsigned char* dst = vs + (p >> 3) * V_ROW + (p & 7) * 16;
      *reinterpret_cast<uint2*>(dst) = make_uint2(v.x, v.y);
      *reinterpret_cast<uint2*>(dst + 8) = make_uint2(v.z, v.w);
    }
  }
}

template <int W>
__global__ __launch_bounds__(64 * W, 2) void k_attn_mfma(BlockDev b, KvDev kv, int layer, int hq, int hkv,
                                                      const bf16_t* __restrict__ q, float* __restrict__ part_o,
                                                      float* __restrict__ part_ml, int nsplit, int tps,
                                                      int q_tiles) {
  constexpr int HD = 128;
  constexpr int NT = 64 * W;
  constexpr int PIECES = (1024 + NT - 1) / NT;   // 16-byte pieces per thread and tile, K and V alike
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* ks = lds;                       // [2][K_TILE_BYTES]
  unsigned char* vs = lds + 2 * K_TILE_BYTES;    // [2][V_TILE_BYTES]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane & 31, lg = lane >> 5;
  const int G = hq / hkv;
  // XCD-aware logical id (hardware ids go round-robin over the 8 XCDs): the query tiles that
  // stream the same keys (same kv head, same split) get consecutive logical ids on one XCD and
  // so share its L2.
  const int total_wg = q_tiles * hkv * b.batch * nsplit;
  const int per_xcd = (total_wg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= total_wg) return;
  const int qt = logical % q_tiles;
  const int kvh = (logical / q_tiles) % hkv;
  const int zz = logical / (q_tiles * hkv);
  const int seq = zz / nsplit, sp = zz % nsplit;
  const int nr = b.n_rows[seq];
  if (!seq_ok(kv, seq, nr, b.rows_per_seq)) return;
  if (qt * (W * 32) >= nr * G) return;                  // no live query column in this workgroup
  const int L = kv.len[seq], total = L + nr;
  const int ntiles = (total + 63) >> 6;
  const int t0 = sp * tps, t1 = min(ntiles, t0 + tps);

  const int qcol = (qt * W + wave) * 32 + lr;
  const bool col_live = qcol < nr * G;
  const int r = col_live ? qcol / G : 0;
  const int h = kvh * G + (col_live ? qcol % G : 0);
  const size_t row = (size_t)seq * b.rows_per_seq + r;
  const size_t item = (row * hq + h) * nsplit + sp;

  if (t0 >= t1) {   // empty split: neutral partial
    if (col_live) {
      f32x4_t z = {0.f, 0.f, 0.f, 0.f};
      for (int i = lg; i < 32; i += 2) *reinterpret_cast<f32x4_t*>(part_o + item * HD + 4 * i) = z;
      if (lg == 0) { part_ml[item * 2] = NEG_BIG; part_ml[item * 2 + 1] = 0.f; }
    }
    return;
  }

  // Q^T fragments: lane = query column, 8 features per k-step at 16*s + 8*lg
  bf16x8_t qf[8];
  {
    const bf16_t* qp = q + (row * hq + h) * HD + 8 * lg;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * s);
  }
  const uint64_t* anc = b.anc + row * b.anc_words;
  const bf16_t* kp = (const bf16_t*)kv.k + kv_plane(layer, kvh, hkv, kv.capacity, HD);
  const bf16_t* vp = (const bf16_t*)kv.v + kv_plane(layer, kvh, hkv, kv.capacity, HD);
  const int64_t base = kv.base[seq];
  const float scale = LOG2E / sqrtf((float)HD);

  uint4 kreg[PIECES], vreg[PIECES];

  f32x16_t oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[i][v] = 0.f;
  float m = NEG_BIG, l = 0.f;

  // K tile t: 64 rows of 256 B, contiguous; V tile t: [128][64], contiguous
  const bf16_t* kt0 = kp + (size_t)base * HD;
  const bf16_t* vt0 = vp + (size_t)(base >> 6) * HD * 64;
  attn_load_tile<W>(kt0 + (size_t)t0 * 64 * HD, vt0 + (size_t)t0 * 64 * HD, tid, kreg, vreg);
  attn_store_tile<W>(ks, vs, tid, total - t0 * 64, kreg, vreg);
  __syncthreads();

  for (int t = t0; t < t1; ++t) {
    const int buf = (t - t0) & 1;
    const bool more = t + 1 < t1;
    {
      const int tn = more ? t + 1 : t;
      attn_load_tile<W>(kt0 + (size_t)tn * 64 * HD, vt0 + (size_t)tn * 64 * HD, tid, kreg, vreg);
    }

    // S^T = K Q^T for the two 32-key blocks of the tile
    f32x16_t sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[kb][v] = 0.f;
    const unsigned char* kbase = ks + buf * K_TILE_BYTES + lr * K_ROW + 16 * lg;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(kbase + kb * 32 * K_ROW + 32 * s);
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[kb], 0, 0, 0);
      }
    }
    // register v of block kb <-> key kb*32 + 8*(v/4) + 4*lg + v%4
    float tmax = NEG_BIG;
    const int key0 = t * 64;
    if (key0 + 64 <= L) {   // tile inside the committed cache: no mask
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          sacc[kb][v] *= scale;
          tmax = fmaxf(tmax, sacc[kb][v]);
        }
    } else {
      const int c_lo = key0 - L;
      const int w0 = (c_lo > 0 ? c_lo : 0) >> 6;
      const uint64_t a0 = w0 < b.anc_words ? anc[w0] : 0ull;
      const uint64_t a1 = w0 + 1 < b.anc_words ? anc[w0 + 1] : 0ull;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int key = key0 + kb * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
          int c = key - L;
          bool valid = c < 0;
          if (c >= 0 && key < total) {
            uint64_t word = (c >> 6) == w0 ? a0 : a1;
            valid = (word >> (c & 63)) & 1ull;
          }
          float sv = valid ? sacc[kb][v] * scale : NEG_BIG;
          sacc[kb][v] = sv;
          tmax = fmaxf(tmax, sv);
        }
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m, tmax);
    const float alpha = exp2f(m - m_new);
    float lsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float sv = sacc[kb][v];
        float p = sv > 0.5f * NEG_BIG ? exp2f(sv - m_new) : 0.f;
        sacc[kb][v] = p;
        lsum += p;
      }
    l = l * alpha + lsum;
    m = m_new;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[i][v] *= alpha;

    // O^T += V^T P^T: k-step (kb, u) takes registers 8u..8u+7 of block kb, i.e. keys
    // kb*32 + 16u + {0, 8} + 4*lg + 0..3
    const unsigned char* vbase = vs + buf * V_TILE_BYTES + lr * V_ROW + 8 * lg;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        bf16x8_t pf;
#pragma unroll
        for (int j = 0; j < 8; ++j) pf[j] = (bf16_t)sacc[kb][8 * u + j];
        const int koff = 2 * (kb * 32 + 16 * u);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const unsigned char* vptr = vbase + db * 32 * V_ROW + koff;
          uint2 lo = *reinterpret_cast<const uint2*>(vptr);
          uint2 hi = *reinterpret_cast<const uint2*>(vptr + 16);
          uint4 packed = make_uint4(lo.x, lo.y, hi.x, hi.y);
          bf16x8_t vf = __builtin_bit_cast(bf16x8_t, packed);
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[db], 0, 0, 0);
        }
      }
    }
    if (more)
      attn_store_tile<W>(ks + (buf ^ 1) * K_TILE_BYTES, vs + (buf ^ 1) * V_TILE_BYTES, tid, total - (t + 1) * 64, kreg,
                         vreg);
    __syncthreads();
  }

  l += __shfl_xor(l, 32, 64);
  if (col_live) {
    // register v of feature block db <-> feature db*32 + 8*(v/4) + 4*lg + v%4
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        f32x4_t o4 = {oacc[db][4 * vq], oacc[db][4 * vq + 1], oacc[db][4 * vq + 2], oacc[db][4 * vq + 3]};
        *reinterpret_cast<f32x4_t*>(part_o + item * HD + db * 32 + 8 * vq + 4 * lg) = o4;
      }
    if (lg == 0) { part_ml[item * 2] = m; part_ml[item * 2 + 1] = l; }
  }
}

// --------------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_attn_merge(BlockDev b, KvDev kv, int hq, int hd, const float* __restrict__ part_o,
                             const float* __restrict__ part_ml, int nsplit, T* __restrict__ out) {
  const int row = blockIdx.x / hq, h = blockIdx.x % hq;
  const int seq = row / b.rows_per_seq, r = row % b.rows_per_seq;
  const int nr = b.n_rows[seq];
  const int d = threadIdx.x;
  T* dst = out + ((size_t)row * hq + h) * hd + d;
  if (!seq_ok(kv, seq, nr, b.rows_per_seq) || r >= nr) {
    *dst = from_f32<T>(0.f);
    return;
  }
  const size_t item0 = ((size_t)row * hq + h) * nsplit;
  float mx = NEG_BIG;
  for (int s = 0; s < nsplit; ++s) mx = fmaxf(mx, part_ml[(item0 + s) * 2]);
  float lt = 0.f, acc = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    float w = exp2f(part_ml[(item0 + s) * 2] - mx);
    lt += part_ml[(item0 + s) * 2 + 1] * w;
    acc += part_o[(item0 + s) * hd + d] * w;
  }
  *dst = from_f32<T>(lt > 0.f ? acc / lt : 0.f);
}

}  // namespace

AttnPlan attn_plan(int batch, int rows_per_seq, int hq, int hkv, int len_bound) {
  // Splits of the key range: enough workgroups for ~1.5 per CU, but no more -- every split
  // writes a partial (m, l, O) per query row and head that the merge kernel reads back -- and
  // at least 3 key tiles of 64 per split.
  AttnPlan p;
  int nt = (len_bound + rows_per_seq + 63) / 64;
  int G = hq / hkv;
  int qtiles = (rows_per_seq * G + 127) / 128;
  int base = qtiles * hkv * batch;
  int want = (384 + base - 1) / base;
  int max_by_len = std::max(1, nt / 3);
  int ns = std::max(1, std::min(std::min(want, max_by_len), 64));
  p.tiles_per_split = (nt + ns - 1) / ns;
  p.nsplit = (nt + p.tiles_per_split - 1) / p.tiles_per_split;
  return p;
}

size_t attn_partial_floats(int batch, int rows_per_seq, int hq, int hd, int nsplit) {
  return (size_t)batch * rows_per_seq * hq * nsplit * (hd + 2);
}

hipError_t launch_attn(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int layer, int hq, int hkv,
                       int hd, const void* q, float* partials, const AttnPlan& p) {
  const int M = b.batch * b.rows_per_seq;
  float* part_o = partials;
  float* part_ml = partials + (size_t)M * hq * p.nsplit * hd;
  if (dtype == ESP_BF16 && hd == 128) {
    const int G = hq / hkv;
    const int cols = b.rows_per_seq * G;
    const int wave_tiles = (cols + 31) / 32;
    // waves per workgroup: the count in 2..4 that pads the column range least (ties: larger)
    int W = 4, best_pad = 1 << 30;
    for (int w = 4; w >= 2; --w) {
      int pad = ((wave_tiles + w - 1) / w) * w - wave_tiles;
      if (pad < best_pad) { best_pad = pad; W = w; }
    }
    const int q_tiles = (wave_tiles + W - 1) / W;
    const int total_wg = q_tiles * hkv * b.batch * p.nsplit;
    dim3 grid(((total_wg + 7) / 8) * 8);
    size_t lds = 2 * (size_t)(K_TILE_BYTES + V_TILE_BYTES);
    // more than 64 KB of dynamic LDS must be granted per kernel once
    static bool lds_granted = false;
    if (!lds_granted) {
      hipError_t e1 = hipSuccess;
      hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_mfma<2>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipError_t e3 = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_mfma<3>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipError_t e4 = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_mfma<4>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e1 != hipSuccess) return e1;
      if (e2 != hipSuccess) return e2;
      if (e3 != hipSuccess) return e3;
      if (e4 != hipSuccess) return e4;
      lds_granted = true;
    }
#define ESP_ATTN_CASE(w)                                                                                  \
  case w:                                                                                                 \
    hipLaunchKernelGGL(k_attn_mfma<w>, grid, dim3(64 * w), lds, st, b, kv, layer, hq, hkv, (const bf16_t*)q, \
                       part_o, part_ml, p.nsplit, p.tiles_per_split, q_tiles);                            \
    break;
    switch (W) {
      ESP_ATTN_CASE(2)
      ESP_ATTN_CASE(3)
      ESP_ATTN_CASE(4)
    }
#undef ESP_ATTN_CASE
  } else {
    dim3 grid(M, hq, p.nsplit);
    if (dtype == ESP_F32 && hd == 64)
      hipLaunchKernelGGL((k_attn_generic<float, 64>), grid, dim3(64), 0, st, b, kv, layer, hq, hkv, (const float*)q,
                         part_o, part_ml, p.nsplit, p.tiles_per_split);
    else if (dtype == ESP_F32 && hd == 128)
      hipLaunchKernelGGL((k_attn_generic<float, 128>), grid, dim3(64), 0, st, b, kv, layer, hq, hkv,
                         (const float*)q, part_o, part_ml, p.nsplit, p.tiles_per_split);
    else if (dtype == ESP_BF16 && hd == 64)
      hipLaunchKernelGGL((k_attn_generic<bf16_t, 64>), grid, dim3(64), 0, st, b, kv, layer, hq, hkv,
                         (const bf16_t*)q, part_o, part_ml, p.nsplit, p.tiles_per_split);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_attn_merge(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int hq, int hd,
                             const float* partials, const AttnPlan& p, void* out) {
  const int M = b.batch * b.rows_per_seq;
  const float* part_o = partials;
  const float* part_ml = partials + (size_t)M * hq * p.nsplit * hd;
  if (dtype == ESP_F32)
    hipLaunchKernelGGL(k_attn_merge<float>, dim3(M * hq), dim3(hd), 0, st, b, kv, hq, hd, part_o, part_ml, p.nsplit,
                       (float*)out);
  else
    hipLaunchKernelGGL(k_attn_merge<bf16_t>, dim3(M * hq), dim3(hd), 0, st, b, kv, hq, hd, part_o, part_ml,
                       p.nsplit, (bf16_t*)out);
  return hipGetLastError();
}
