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
      float acc = 0.f;
      for (int d = 0; d < HD; ++d) acc = fmaf(to_f32(kp[k_off(base + key, d, HD)]), qs[d], acc);
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
      for (int kk = 0; kk < nk; ++kk) a = fmaf(ps[kk], to_f32(vp[v_off(base + t * 64 + kk, lane + 64 * i, HD)]), a);
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
constexpr int K_TILE_BYTES = 64 * 128 * 2;   // 64 keys: two cache blocks of 32 slots, 16 fragments of 1 KB
constexpr int V_TILE_BYTES = 64 * 128 * 2;

// Tile staging: a tile of 64 keys is 16 KB of K and 16 KB of V, both contiguous in the cache and
// already in fragment order, so staging is a linear copy.  Loads are unconditional (a piece index
// past the tile is clamped and its value dropped at the store) so the staging registers stay in
// VGPRs.
template <int W>
__device__ __forceinline__ void attn_load_tile(const bf16_t* __restrict__ kt, const bf16_t* __restrict__ vt, int tid,
                                               u32x4_t (&kreg)[(1024 + 64 * W - 1) / (64 * W)],
                                               u32x4_t (&vreg)[(1024 + 64 * W - 1) / (64 * W)]) {
  constexpr int NT = 64 * W, PIECES = (1024 + NT - 1) / NT;
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    int p = min(tid + NT * i, 1023);
    kreg[i] = *reinterpret_cast<const u32x4_t*>(kt + (size_t)p * 8);
    vreg[i] = *reinterpret_cast<const u32x4_t*>(vt + (size_t)p * 8);
  }
}

template <int W, bool LAST>
__device__ __forceinline__ void attn_store_pieces(unsigned char* ks, unsigned char* vs, int tid, int keys_left,
                                                  const u32x4_t (&kreg)[(1024 + 64 * W - 1) / (64 * W)],
                                                  const u32x4_t (&vreg)[(1024 + 64 * W - 1) / (64 * W)]) {
  constexpr int NT = 64 * W, PIECES = (1024 + NT - 1) / NT;
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    int p = tid + NT * i;
    if (1024 % NT == 0 || p < 1024) {
      *reinterpret_cast<u32x4_t*>(ks + p * 16) = kreg[i];
      u32x4_t v = vreg[i];
      if (LAST) {
        // piece p = fragment (block p/512, key-step (p/64)%2) of lane p%64; word w holds elements
        // 2w, 2w+1 = keys k0, k0+1
        const int kbase = (p >> 9) * 32 + ((p >> 6) & 1) * 16 + ((p >> 5) & 1) * 4;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int k0 = kbase + 8 * (w >> 1) + 2 * (w & 1);
          v[w] &= k0 + 1 < keys_left ? 0xffffffffu : (k0 < keys_left ? 0x0000ffffu : 0u);
        }
      }
      *reinterpret_cast<u32x4_t*>(vs + p * 16) = v;
    }
  }
}

// keys_left: keys of the tile that belong to the sequence; V of the others is zeroed (their
// probability is zero, but 0 * NaN from never-written cache memory would poison the MFMA).
// Only the last tile of a sequence takes that path (one uniform branch).
template <int W>
__device__ __forceinline__ void attn_store_tile(unsigned char* ks, unsigned char* vs, int tid, int keys_left,
                                                const u32x4_t (&kreg)[(1024 + 64 * W - 1) / (64 * W)],
                                                const u32x4_t (&vreg)[(1024 + 64 * W - 1) / (64 * W)]) {
  if (keys_left < 64) attn_store_pieces<W, true>(ks, vs, tid, keys_left, kreg, vreg);
  else attn_store_pieces<W, false>(ks, vs, tid, keys_left, kreg, vreg);
}

// Visibility bits of 64 consecutive keys for one block row: bit j stands for block position
// c_lo + j (negative positions are committed cache slots, always visible; positions from
// keys_in_tile on lie past the sequence).  anc is the row's ancestor bitset.
__device__ __forceinline__ uint64_t key_window(const uint64_t* __restrict__ anc, int anc_words, int c_lo,
                                               int keys_in_tile) {
  uint64_t wnd;
  if (c_lo < 0) {
    const int n = -c_lo;                                   // 1..63 cache keys lead the tile
    const uint64_t a0 = anc_words > 0 ? anc[0] : 0ull;
    wnd = (a0 << n) | ((1ull << n) - 1ull);
  } else {
    const int w0 = c_lo >> 6, sh = c_lo & 63;
    const uint64_t a0 = w0 < anc_words ? anc[w0] : 0ull;
    const uint64_t a1 = w0 + 1 < anc_words ? anc[w0 + 1] : 0ull;
    wnd = sh ? (a0 >> sh) | (a1 << (64 - sh)) : a0;
  }
  if (keys_in_tile < 64) wnd &= (1ull << keys_in_tile) - 1ull;
  return wnd;
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

  u32x4_t kreg[PIECES], vreg[PIECES];

  f32x16_t oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[i][v] = 0.f;
  float m = NEG_BIG, l = 0.f;

  // tile t of K and of V: 64 * HD elements each, contiguous (two cache blocks)
  const bf16_t* kt0 = kp + (size_t)base * HD;
  const bf16_t* vt0 = vp + (size_t)base * HD;
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

    // S^T = K Q^T for the two 32-key blocks of the tile.  The MFMA phases run at raised wave
    // priority: of the two waves that share a SIMD, the one with matrix work issues first and the
    // other fills the gaps with its softmax arithmetic.
    __builtin_amdgcn_s_setprio(2);
    f32x16_t sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[kb][v] = 0.f;
    // Fragment reads run one group (4 reads, 4 MFMAs) ahead of their use and are pinned there by
    // scheduling barriers: left to itself the compiler funnels every read through one register
    // quad and waits out the full LDS latency before each MFMA.
    const unsigned char* kbase = ks + buf * K_TILE_BYTES + lane * 16;   // fragment (kb, s) at (kb*8 + s) KB
    bf16x8_t fr[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j)   // group g holds steps 2g, 2g+1 of both key blocks: j = 2*(s&1) + kb
      fr[0][j] = *reinterpret_cast<const bf16x8_t*>(kbase + ((j & 1) * 8 + (j >> 1)) * 1024);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (g < 3) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          fr[(g + 1) & 1][j] =
              *reinterpret_cast<const bf16x8_t*>(kbase + ((j & 1) * 8 + 2 * (g + 1) + (j >> 1)) * 1024);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        sacc[j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g & 1][j], qf[2 * g + (j >> 1)], sacc[j & 1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // register v of block kb <-> key kb*32 + 8*(v/4) + 4*lg + v%4.  Scores stay unscaled; the
    // scale is folded into the exponent: p = 2^(s*scale - m*scale).
    const int key0 = t * 64;
    const bool masked_tile = key0 + 64 > L;   // tiles inside the committed cache need no mask
    if (masked_tile) {
      // visibility of the tile's 64 keys for this lane's row, bit j <-> key key0 + j
      const uint64_t wnd = key_window(anc, b.anc_words, key0 - L, total - key0);
      const unsigned wlo = (unsigned)wnd >> (4 * lg), whi = (unsigned)(wnd >> 32) >> (4 * lg);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const unsigned bit = ((kb ? whi : wlo) >> (8 * (v >> 2) + (v & 3))) & 1u;
          sacc[kb][v] = bit ? sacc[kb][v] : NEG_BIG;
        }
    }
    __builtin_amdgcn_s_setprio(0);
    float tmax = NEG_BIG;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sacc[kb][v]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m, tmax);
    const float mb = m_new * scale;
    if (__builtin_amdgcn_ballot_w64(m_new > m) != 0ull) {   // rescale only when some column's max moved
      const float alpha = __builtin_amdgcn_exp2f(m * scale - mb);
      l *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[i][v] *= alpha;
    }
    m = m_new;
    float lsum = 0.f;
    if (masked_tile) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float sv = sacc[kb][v];
          float p = sv > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(fmaf(sv, scale, -mb)) : 0.f;
          sacc[kb][v] = p;
          lsum += p;
        }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][v], scale, -mb));
          sacc[kb][v] = p;
          lsum += p;
        }
    }
    l += lsum;

    // O^T += V^T P^T: k-step (kb, u) takes registers 8u..8u+7 of block kb, i.e. keys
    // kb*32 + 16u + {0, 8} + 4*lg + 0..3 -- one 16-byte read in the permuted LDS order
    __builtin_amdgcn_s_setprio(2);
    const unsigned char* vbase = vs + buf * V_TILE_BYTES + lane * 16;   // fragment (kb, db, u) at (kb*8 + db*2 + u) KB
#pragma unroll
    for (int db = 0; db < 4; ++db) fr[0][db] = *reinterpret_cast<const bf16x8_t*>(vbase + db * 2048);
#pragma unroll
    for (int ku = 0; ku < 4; ++ku) {   // k-step ku = 2*kb + u
      if (ku < 3) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
          fr[(ku + 1) & 1][db] =
              *reinterpret_cast<const bf16x8_t*>(vbase + (((ku + 1) >> 1) * 8 + db * 2 + ((ku + 1) & 1)) * 1024);
      }
      bf16x8_t pf;
#pragma unroll
      for (int j = 0; j < 8; ++j) pf[j] = (bf16_t)sacc[ku >> 1][8 * (ku & 1) + j];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int db = 0; db < 4; ++db)
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[ku & 1][db], pf, oacc[db], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_setprio(0);
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
    if (lg == 0) { part_ml[item * 2] = m * scale; part_ml[item * 2 + 1] = l; }   // m in the exponent's units
  }
}

// --------------------------------------------------------------------------------------------------
__device__ __forceinline__ void store4(float* dst, f32x4_t v) { *reinterpret_cast<f32x4_t*>(dst) = v; }
__device__ __forceinline__ void store4(bf16_t* dst, f32x4_t v) {
  bf16x4_t o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
  *reinterpret_cast<bf16x4_t*>(dst) = o;
}

// Merge of the per-split partials, in split order.  hd/4 threads per (row, head) item, four
// features each; a 256-thread workgroup takes 256/(hd/4) items.
template <typename T>
__global__ __launch_bounds__(256) void k_attn_merge(BlockDev b, KvDev kv, int hq, int hd,
                                                    const float* __restrict__ part_o,
                                                    const float* __restrict__ part_ml, int nsplit,
                                                    T* __restrict__ out, int n_items) {
  const int per = hd >> 2;
  const int item = blockIdx.x * (256 / per) + threadIdx.x / per;   // row * hq + h
  const int d = (threadIdx.x % per) * 4;
  if (item >= n_items) return;
  const int row = item / hq;
  const int seq = row / b.rows_per_seq, r = row % b.rows_per_seq;
  const int nr = b.n_rows[seq];
  T* dst = out + (size_t)item * hd + d;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  if (!seq_ok(kv, seq, nr, b.rows_per_seq) || r >= nr) {
    store4(dst, acc);
    return;
  }
  const size_t item0 = (size_t)item * nsplit;
  float mx = NEG_BIG;
  for (int s = 0; s < nsplit; ++s) mx = fmaxf(mx, part_ml[(item0 + s) * 2]);
  float lt = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float w = exp2f(part_ml[(item0 + s) * 2] - mx);
    lt += part_ml[(item0 + s) * 2 + 1] * w;
    const f32x4_t o = *reinterpret_cast<const f32x4_t*>(part_o + (item0 + s) * hd + d);
    acc += o * w;
  }
  const float inv = lt > 0.f ? 1.f / lt : 0.f;
  store4(dst, acc * inv);
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
    // waves per workgroup: 3 or 4, whichever pads the column range less (ties: 4)
    int W = 4, best_pad = 1 << 30;
    for (int w = 4; w >= 3; --w) {
      int pad = ((wave_tiles + w - 1) / w) * w - wave_tiles;
      if (pad < best_pad) { best_pad = pad; W = w; }
    }
    const int q_tiles = (wave_tiles + W - 1) / W;
    const int total_wg = q_tiles * hkv * b.batch * p.nsplit;
    dim3 grid(((total_wg + 7) / 8) * 8);
    size_t lds = 2 * (size_t)(K_TILE_BYTES + V_TILE_BYTES);
    // 64 KB of dynamic LDS: the default limit, no attribute needed
#define ESP_ATTN_CASE(w)                                                                                  \
  case w:                                                                                                 \
    hipLaunchKernelGGL(k_attn_mfma<w>, grid, dim3(64 * w), lds, st, b, kv, layer, hq, hkv, (const bf16_t*)q, \
                       part_o, part_ml, p.nsplit, p.tiles_per_split, q_tiles);                            \
    break;
    switch (W) {
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
  const int n_items = M * hq, per_wg = 256 / (hd / 4);
  const dim3 grid((n_items + per_wg - 1) / per_wg);
  if (dtype == ESP_F32)
    hipLaunchKernelGGL(k_attn_merge<float>, grid, dim3(256), 0, st, b, kv, hq, hd, part_o, part_ml, p.nsplit,
                       (float*)out, n_items);
  else
    hipLaunchKernelGGL(k_attn_merge<bf16_t>, grid, dim3(256), 0, st, b, kv, hq, hd, part_o, part_ml, p.nsplit,
                       (bf16_t*)out, n_items);
  return hipGetLastError();
}
