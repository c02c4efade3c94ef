// Tree-masked grouped-query attention of one decoder layer (paper Sec. 3.3, App. C, App. E).
//
// Row r of sequence b attends to cache slots [0, len[b]) and to the block rows c whose bit is set
// in its ancestor bitset (held at slots len[b] + c).  Only the last n_rows keys of a sequence need
// a mask test; every tile that lies inside the committed cache runs unmasked.
//
// bf16 / head_dim 128 path (k_attn_ring, described at its definition): the G = n_q/n_kv query heads
// of a kv head times the block rows form the "query columns" of a (keys x queries) problem; a
// workgroup owns the columns of one kv head and one split of the key range, and the per-split partial
// (m, l, O) are merged by k_attn_merge_ring in split order (fixed, so results do not depend on
// scheduling).
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
// k_attn_ring: the bf16 / head_dim 128 kernel.
//
// One workgroup per CU owns up to 384 query columns (query row x head of one kv group; a wave per
// 32 columns, 4 to 12 waves, so two to three waves share a SIMD and the softmax arithmetic of one
// overlaps the matrix work of another) and one split of the key range.  K/V tiles of 64 keys
// (16 KB + 16 KB, already in fragment order in the cache) go from global memory straight into a
// ring of four LDS stages (no register hop, up to three tiles in flight) and are shared by all the
// waves.  S^T = K Q^T and O^T = V^T P^T both run on v_mfma_f32_32x32x16_bf16: computing the
// transposed scores leaves each lane with one query column and 16 keys per 32-key block, which is
// exactly the B-operand layout P^T needs, so the probabilities never leave registers.  Online
// softmax in fp32 (base-2 exponent), one exchange between the two lane halves per 32 keys.
// Partial (m, l, O) per split are merged by k_attn_merge_ring in split order (fixed, so results do
// not depend on scheduling).
constexpr int K_TILE_BYTES = 64 * 128 * 2;   // 64 keys: two cache blocks of 32 slots, 16 fragments of 1 KB
constexpr int V_TILE_BYTES = 64 * 128 * 2;
constexpr int RING_STAGES = 4;
constexpr int STAGE_BYTES = K_TILE_BYTES + V_TILE_BYTES;
constexpr int RING_LDS_BYTES = RING_STAGES * STAGE_BYTES;
constexpr int RING_MAX_WAVES = 12;
// The reference m of a column's exponents follows its running maximum lazily: it is set by the first
// unit that has a visible key and moves only when a score exceeds it by more than this many powers of
// two, so the output accumulators are rescaled a few times per split instead of at almost every unit.
// Probabilities may reach 2^RESCALE_SLACK, which fp32 sums and the bf16 operand of the P V product
// hold without loss of relative precision.
constexpr float RESCALE_SLACK = 24.0f;

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

// zeroes, in the LDS copy of the sequence's last tile, the V entries of keys past its end (their
// probability is zero, but 0 * NaN from never-written cache memory would poison the accumulators)
__device__ __forceinline__ void ring_zero_tail(unsigned char* vs, int keys_left, int tid, int nthreads) {
  for (int p = tid; p < 1024; p += nthreads) {
    u32x4_t v = *reinterpret_cast<u32x4_t*>(vs + p * 16);
    // piece p = fragment (block p/512, key-step (p/64)%2) of lane p%64; word w holds elements
    // 2w, 2w+1 = keys k0, k0+1
    const int kbase = (p >> 9) * 32 + ((p >> 6) & 1) * 16 + ((p >> 5) & 1) * 4;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int k0 = kbase + 8 * (w >> 1) + 2 * (w & 1);
      v[w] &= k0 + 1 < keys_left ? 0xffffffffu : (k0 < keys_left ? 0x0000ffffu : 0u);
    }
    *reinterpret_cast<u32x4_t*>(vs + p * 16) = v;
  }
}

// max of a value with the value held by the lane 32 places away (the other half of the wave holds the
// other 16 keys of the same column): one v_permlane32_swap (swaps the upper half of its first operand
// with the lower half of its second; given the value twice, each result holds one half's values in
// both halves) instead of a round trip through the LDS crossbar
__device__ __forceinline__ float max_across_halves(float v) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// One unit of 32 keys for the wave's 32 columns: scores, online softmax, P V.
// kst / vst: this lane's 16 bytes of the unit's first K fragment (step s at + s KB) and first V
// fragment ((db, u) at + (db * 2 + u) KB).  vis: visibility bits of this lane's 16 keys at bit
// 8 (v / 4) + v % 4 (register v <-> key 8 (v / 4) + 4 half + v % 4), used when `masked` (wave-uniform).
__device__ __forceinline__ void ring_unit(bool masked, const unsigned char* kst, const unsigned char* vst, unsigned vis, float scale,
                                          const bf16x8_t (&qf)[8], f32x16_t (&oacc)[4], float& m, float& l) {
  f32x16_t sc;
#pragma unroll
  for (int v = 0; v < 16; ++v) sc[v] = 0.f;
  // fragment reads run one step ahead of their MFMA and are pinned there (scheduling barriers): left
  // to itself the compiler hoists all of them and runs out of registers
  // the matrix phases run at raised wave priority: of the waves that share a SIMD, one with matrix
  // work issues first and the others fill the gaps with their softmax arithmetic
  // (the LDS answers after three to four MFMA times: PF reads are in flight, as many as the
  // registers allow)
  constexpr int PF = 3, NF = PF + 1;
  bf16x8_t fr[NF];
  // fragment j of the unit's 16: K steps 0..7, then V fragments in the order (u, db) = j - 8
  auto frag_at = [&](int j) {
    return j < 8 ? *reinterpret_cast<const bf16x8_t*>(kst + j * 1024)
                 : *reinterpret_cast<const bf16x8_t*>(vst + ((((j - 8) & 3) * 2) + ((j - 8) >> 2)) * 1024);
  };
#pragma unroll
  for (int j = 0; j < PF; ++j) fr[j] = frag_at(j);
  __builtin_amdgcn_s_setprio(2);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    fr[(s + PF) % NF] = frag_at(s + PF);
    __builtin_amdgcn_sched_barrier(0);
    sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[s % NF], qf[s], sc, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_setprio(0);
  // scores stay unscaled; the scale is folded into the exponent: p = 2^(s*scale - m*scale)
  if (masked) {
#pragma unroll
    for (int v = 0; v < 16; ++v) sc[v] = ((vis >> (8 * (v >> 2) + (v & 3))) & 1u) ? sc[v] : NEG_BIG;
  }
  float tmax = fmaxf(sc[0], sc[1]);
#pragma unroll
  for (int v = 2; v < 16; v += 2) tmax = fmaxf(tmax, fmaxf(sc[v], sc[v + 1]));
  tmax = max_across_halves(tmax);
  const float m_new = tmax * scale > m * scale + RESCALE_SLACK ? tmax : m;
  // no key of the column visible so far (m_new at its start value): any finite reference does, the
  // masked scores' exponents then lie far below the range and their probabilities come out as 0
  const float mb = m_new > 0.5f * NEG_BIG ? m_new * scale : 0.f;
  // m still at its start value: nothing accumulated yet, nothing to scale
  const bool moved = m_new != m && m > 0.5f * NEG_BIG;
  if (__builtin_amdgcn_ballot_w64(moved) != 0ull) {
    const float alpha = m > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f(m * scale - mb) : 1.0f;
    l *= alpha;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[i][v] *= alpha;
  }
  m = m_new;
  __builtin_amdgcn_sched_barrier(0);
  // exponentials four at a time (fenced: all sixteen in flight at once cost registers the Q
  // fragments need), converted to the bf16 operand fragments as they come
  float lsum = 0.f;
  bf16x8_t pf[2];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int v = 4 * c + e;
      // a masked score is NEG_BIG: its exponent lies far below the range, p = 0 without a test
      float p = __builtin_amdgcn_exp2f(fmaf(sc[v], scale, -mb));
      lsum += p;
      pf[v >> 3][v & 7] = (bf16_t)p;
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  l += lsum;
  __builtin_amdgcn_s_setprio(2);
  // O^T += V^T P^T: k-step u takes registers 8u..8u+7, i.e. keys 16u + {0, 8} + 4 half + 0..3 -- one
  // 16-byte read in the permuted LDS order
#pragma unroll
  for (int i = 0; i < 8; ++i) {                 // i = u * 4 + db
    const int u = i >> 2, db = i & 3;
    if (i + PF < 8) fr[(8 + i + PF) % NF] = frag_at(8 + i + PF);
    __builtin_amdgcn_sched_barrier(0);
    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[(8 + i) % NF], pf[u], oacc[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_setprio(0);
}

// LPW: 1 KB wave-loads per loading wave and tile (the first 32 / LPW waves of the workgroup load)
template <int LPW>
__global__ __launch_bounds__(64 * RING_MAX_WAVES) void k_attn_ring(BlockDev b, KvDev kv, int layer, int hq, int hkv,
                                                                  const bf16_t* __restrict__ q,
                                                                  float* __restrict__ part_o,
                                                                  float* __restrict__ part_ml, int nsplit, int tps,
                                                                  int q_tiles, int ct_wg, int n_full) {
  constexpr int HD = 128;
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lg = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // this wave's column tile inside the workgroup and the halves of every key tile it works on: waves
  // up to n_full take a whole tile each, the others pair up on one (first = keys 0..31 of a tile,
  // second = keys 32..63) and are merged at the end; waves beyond the tiles only help load
  const int ctl = wave < n_full ? wave : n_full + ((wave - n_full) >> 1);
  const bool pair = wave >= n_full;
  const int kh_first = pair ? ((wave - n_full) & 1) : 0, kh_last = pair ? kh_first : 1;
  const int G = hq / hkv;
  // XCD-aware logical id: the query tiles that stream the same keys (same kv head, same split) get
  // consecutive logical ids on one XCD and so share its L2
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
  const int ncols = nr * G;
  if (qt * ct_wg * 32 >= ncols) return;                 // no live query column in this workgroup
  const int L = kv.len[seq], total = L + nr;
  const int ntiles = (total + 63) >> 6;
  const int t0 = sp * tps, t1 = min(ntiles, t0 + tps);
  const int nt = t1 - t0;

  const int qcol = (qt * ct_wg + ctl) * 32 + lr;
  const bool col_live = qcol < ncols;
  const bool wave_live = ctl < ct_wg && (qt * ct_wg + ctl) * 32 < ncols;  // wave-uniform
  const int r = col_live ? qcol / G : 0;
  const int h = kvh * G + (col_live ? qcol % G : 0);
  const size_t row = (size_t)seq * b.rows_per_seq + r;
  // partial of this wave's column tile and split: O^T as [feature][column] (a store instruction of
  // the wave covers whole 128-byte lines), then (m, l) per column
  const size_t ptile = (((size_t)seq * hkv + kvh) * (q_tiles * ct_wg) + qt * ct_wg + min(ctl, ct_wg - 1)) * nsplit + sp;
  float* po = part_o + ptile * (HD * 32);
  float* pml = part_ml + ptile * 64;

  if (nt <= 0) {   // empty split: neutral partial
    if (wave_live && kh_first == 0) {
      for (int f = lg; f < HD; f += 2) po[f * 32 + lr] = 0.f;
      if (lg == 0) { pml[lr * 2] = NEG_BIG; pml[lr * 2 + 1] = 0.f; }
    }
    return;
  }

  // ---- ring: tile i of the split lives in stage i % 4; piece p of a tile (1 KB) is K piece p for
  // p < 16, V piece p - 16 otherwise; loading wave w brings pieces w * LPW .. w * LPW + LPW - 1
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  const bool loader = wave < 32 / LPW;
  const int64_t base = kv.base[seq];
  const unsigned char* kt0 =
      reinterpret_cast<const unsigned char*>((const bf16_t*)kv.k + kv_plane(layer, kvh, hkv, kv.capacity, HD) + (size_t)base * HD);
  const unsigned char* vt0 =
      reinterpret_cast<const unsigned char*>((const bf16_t*)kv.v + kv_plane(layer, kvh, hkv, kv.capacity, HD) + (size_t)base * HD);
  const int piece0 = wave * LPW;                        // wave-uniform
  const unsigned char* src0 = (piece0 < 16 ? kt0 : vt0) + (size_t)(piece0 & 15) * 1024;
  const uint32_t lane_off = (uint32_t)lane * 16;
  auto issue_tile = [&](int i) {
    if (!loader) return;
    const unsigned char* src = src0 + (size_t)(t0 + i) * K_TILE_BYTES;
    const uint32_t dst = lds0 + (i & 3) * STAGE_BYTES + piece0 * 1024;
    load_to_lds16_sbase<0>(src, lane_off, dst);
    load_to_lds16_sbase<1024>(src, lane_off, dst);
    load_to_lds16_sbase<2048>(src, lane_off, dst);
    load_to_lds16_sbase<3072>(src, lane_off, dst);
    if (LPW == 8) {
      load_to_lds16_sbase<0>(src + 4096, lane_off, dst + 4096);
      load_to_lds16_sbase<1024>(src + 4096, lane_off, dst + 4096);
      load_to_lds16_sbase<2048>(src + 4096, lane_off, dst + 4096);
      load_to_lds16_sbase<3072>(src + 4096, lane_off, dst + 4096);
    }
  };
  // Q^T fragments: lane = query column, 8 features per k-step at 16 s + 8 lg.  The compiler places
  // waits on the load counter for the loads it knows of, and one of those inside the tile loop would
  // also drain the ring's prefetches (which it does not know of).  So the fragments are loaded
  // between the first tile's loads and the others', and an empty statement that names them right
  // after makes the compiler wait for them here: by then the first tile (older, loads retire in
  // order) has landed too, which the first iteration needs anyway, and no load of the compiler's is
  // left in flight when the loop starts.
  issue_tile(0);
  bf16x8_t qf[8];
  {
    const bf16_t* qp = q + (row * hq + h) * HD + 8 * lg;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * s);
    asm volatile("" : "+v"(qf[0]), "+v"(qf[1]), "+v"(qf[2]), "+v"(qf[3]), "+v"(qf[4]), "+v"(qf[5]), "+v"(qf[6]), "+v"(qf[7])
                 :: "memory");
  }
  if (nt > 1) issue_tile(1);
  if (nt > 2) issue_tile(2);
  const uint64_t* anc = b.anc + row * b.anc_words;
  const float scale = LOG2E / sqrtf((float)HD);
  f32x16_t oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[i][v] = 0.f;
  float m = NEG_BIG, l = 0.f;

  const unsigned char* frag = lds + lane * 16;          // this lane's 16 bytes of fragment 0 of stage 0
  for (int i = 0; i < nt; ++i) {
    // tile i has landed (this wave's loads: they retire in order and the tiles after i stay in
    // flight; the barrier covers the other waves'); every wave is done with tile i - 1, whose stage
    // takes tile i + 3
    if (i + 2 < nt) wait_loads_but<2 * LPW>();
    else if (i + 1 < nt) wait_loads_but<LPW>();
    else wait_loads_but<0>();
    __syncthreads();
    if (i + 3 < nt) issue_tile(i + 3);
    const int key0 = (t0 + i) * 64;
    const int keys_left = total - key0;
    if (keys_left < 64) {
      ring_zero_tail(lds + (i & 3) * STAGE_BYTES + K_TILE_BYTES, keys_left, tid, blockDim.x);
      __syncthreads();
    }
    if (!wave_live) continue;
    const unsigned char* st = frag + (i & 3) * STAGE_BYTES;
    const bool masked = key0 + 64 > L;                   // the tile touches the block rows or the sequence's end
    uint64_t wnd = 0;
    if (masked) wnd = key_window(anc, b.anc_words, key0 - L, keys_left);
    if (kh_first == 0) ring_unit(masked, st, st + K_TILE_BYTES, (unsigned)wnd >> (4 * lg), scale, qf, oacc, m, l);
    if (kh_last == 1)
      ring_unit(masked, st + 8192, st + K_TILE_BYTES + 8192, (unsigned)(wnd >> 32) >> (4 * lg), scale, qf, oacc, m, l);
  }

  l += __shfl_xor(l, 32, 64);
  if (n_full < ct_wg) {
    // paired waves: the second hands its (m, l, O) to the first through LDS (the ring is free now)
    __syncthreads();
    float* xo = reinterpret_cast<float*>(lds) + (size_t)(ctl - n_full) * (HD * 32 + 64);
    if (pair && kh_first == 1 && wave_live) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) xo[(db * 16 + v) * 64 + lane] = oacc[db][v];
      if (lg == 0) { xo[HD * 32 + lr * 2] = m; xo[HD * 32 + lr * 2 + 1] = l; }
    }
    __syncthreads();
    if (pair && kh_first == 0 && wave_live) {
      const float mo = xo[HD * 32 + lr * 2], lo = xo[HD * 32 + lr * 2 + 1];
      const float mm = fmaxf(m, mo);
      // a side that saw no visible key (m at its start value) holds nothing: weight it out
      const float wa = m > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f((m - mm) * scale) : 0.f;
      const float wb = mo > 0.5f * NEG_BIG ? __builtin_amdgcn_exp2f((mo - mm) * scale) : 0.f;
      l = l * wa + lo * wb;
      m = mm;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = oacc[db][v] * wa + xo[(db * 16 + v) * 64 + lane] * wb;
    }
  }
  if (wave_live && kh_first == 0) {
    // register v of feature block db <-> feature db*32 + 8*(v/4) + 4*lg + v%4
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) po[(db * 32 + 8 * (v >> 2) + 4 * lg + (v & 3)) * 32 + lr] = oacc[db][v];
    if (lg == 0) { pml[lr * 2] = m * scale; pml[lr * 2 + 1] = l; }   // m in the exponent's units
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

// Merge for the ring kernel's partial layout ([column tile][split][feature][column]), in split
// order.  A workgroup of 256 threads takes 32 features of one column tile of 32 query columns.
// First the weights 2^(m_s - max) of the tile's columns and splits: thread (split group, column)
// fetches the (m, l) of every eighth split at once -- one after the other, a column's splits would
// cost a memory latency each -- and the eight groups combine through LDS.  Then thread (column,
// feature quad) sums the splits' O, every load instruction of a wave covering whole 128-byte lines.
template <int MAXS>
__global__ __launch_bounds__(256) void k_attn_merge_ring(BlockDev b, KvDev kv, int hq, int hkv,
                                                         const float* __restrict__ part_o,
                                                         const float* __restrict__ part_ml, int nsplit,
                                                         int n_ct, bf16_t* __restrict__ out) {
  constexpr int HD = 128, PER = MAXS / 8;
  __shared__ float w_s[MAXS][32];
  __shared__ float red[8][32];
  __shared__ float red_l[8][32];
  const int G = hq / hkv;
  const int fq = blockIdx.x & 3;
  const int tile = blockIdx.x >> 2;                 // (seq * hkv + kvh) * n_ct + ct
  const int ct = tile % n_ct, kvh = (tile / n_ct) % hkv, seq = tile / (n_ct * hkv);
  const int nr = b.n_rows[seq];
  const bool ok = seq_ok(kv, seq, nr, b.rows_per_seq);
  const int col = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int c = ct * 32 + col;                      // column within the kv group
  const bool in_block = c < b.rows_per_seq * G;     // has an output row at all
  const bool live = ok && c < nr * G;
  const size_t t0 = (size_t)tile * nsplit;
  float ms[PER], ls[PER];
  float mx = NEG_BIG;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int sp = grp + 8 * i;
    ms[i] = NEG_BIG; ls[i] = 0.f;
    if (live && sp < nsplit) {
      const float2 ml = *reinterpret_cast<const float2*>(part_ml + (t0 + sp) * 64 + col * 2);
      ms[i] = ml.x; ls[i] = ml.y;
    }
    mx = fmaxf(mx, ms[i]);
  }
  red[grp][col] = mx;
  __syncthreads();
#pragma unroll
  for (int g = 0; g < 8; ++g) mx = fmaxf(mx, red[g][col]);
  float lt = 0.f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int sp = grp + 8 * i;
    const float w = exp2f(ms[i] - mx);
    if (sp < nsplit) w_s[sp][col] = w;
    lt += ls[i] * w;
  }
  red_l[grp][col] = lt;
  __syncthreads();
  if (!in_block) return;
  // the splits' sums are added in group order: fixed, like everything else here
  lt = 0.f;
#pragma unroll
  for (int g = 0; g < 8; ++g) lt += red_l[g][col];
  const float inv = lt > 0.f ? 1.f / lt : 0.f;
  const int fsub = grp;
  const int f0 = fq * 32 + fsub * 4;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  if (live) {
    const float* p = part_o + t0 * (HD * 32) + (size_t)f0 * 32 + col;
#pragma unroll 8
    for (int s = 0; s < nsplit; ++s) {
      const float w = w_s[s][col];
      const float* ps = p + (size_t)s * (HD * 32);
      acc[0] += ps[0] * w; acc[1] += ps[32] * w; acc[2] += ps[64] * w; acc[3] += ps[96] * w;
    }
    acc *= inv;
  }
  const int r = c / G, h = kvh * G + c % G;
  store4(out + (((size_t)seq * b.rows_per_seq + r) * hq + h) * HD + f0, acc);
}

}  // namespace

// the ring kernel uses more dynamic LDS than a kernel gets by default: raise the limit once (also
// called when a context is created, so that no launch inside a stream capture is the first one)
hipError_t attn_prepare() {
  static const hipError_t attr = [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_ring<4>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, RING_LDS_BYTES);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_ring<8>), hipFuncAttributeMaxDynamicSharedMemorySize,
                               RING_LDS_BYTES);
  }();
  return attr;
}

namespace {
// Geometry of the ring kernel for `cols` query columns per kv head.  A column tile is 32 columns; a
// workgroup owns ct_wg of them (as few workgroups per kv head and split as twelve waves allow, the
// tiles spread evenly).  Its first n_full tiles get a wave each; each of the others is worked by two
// waves, one per half of every key tile, when that evens out the load of the four SIMDs (waves go
// to SIMDs round-robin, and the SIMD with the most matrix work sets the pace): ct_wg = 9 gives
// SIMD loads of 5, 5, 4, 4 half-tiles instead of 6, 4, 4, 4.  At least four waves (they carry the loads).
struct RingGeometry { int q_tiles, ct_wg, n_full, waves; };
RingGeometry ring_geometry(int cols) {
  RingGeometry g;
  const int ct = (cols + 31) / 32;
  g.q_tiles = (ct + RING_MAX_WAVES - 1) / RING_MAX_WAVES;
  g.ct_wg = (ct + g.q_tiles - 1) / g.q_tiles;
  const int rem = g.ct_wg & 3;
  const int n_split = ((rem == 1 || rem == 2) && g.ct_wg > 4 && g.ct_wg + rem <= RING_MAX_WAVES) ? rem : 0;
  g.n_full = g.ct_wg - n_split;
  g.waves = std::max(4, g.n_full + 2 * n_split);
  return g;
}
}  // namespace

AttnPlan attn_plan(int batch, int rows_per_seq, int hq, int hkv, int len_bound) {
  // Splits of the key range.  A workgroup (one per CU) owns the query columns of one kv head -- or a
  // share of them when they exceed twelve waves -- and one split; every split writes a partial
  // (m, l, O) per query row and head that the merge kernel reads back, so: as few splits as fill the
  // 256 CUs once, no second, mostly empty round, and a few tiles of 64 keys per split at least.
  // Cost model per candidate: rounds over the CUs times (tiles per split + a fixed per-workgroup
  // cost of about four tiles).
  AttnPlan p;
  const int nt = (len_bound + rows_per_seq + 63) / 64;
  const int G = hq / hkv;
  const int base = ring_geometry(rows_per_seq * G).q_tiles * hkv * batch;
  int best = 1, best_cost = 1 << 30;
  for (int ns = 1; ns <= 64; ++ns) {
    const int tps = (nt + ns - 1) / ns;
    if (ns > 1 && tps < 2) break;
    if ((nt + tps - 1) / tps != ns) continue;             // same partition as a smaller count
    const int rounds = (base * ns + 255) / 256;
    const int cost = rounds * (tps + 4);
    if (cost < best_cost) { best_cost = cost; best = ns; }
  }
  p.tiles_per_split = (nt + best - 1) / best;
  p.nsplit = (nt + p.tiles_per_split - 1) / p.tiles_per_split;
  return p;
}

size_t attn_partial_floats(int dtype, int batch, int rows_per_seq, int hq, int hkv, int hd, int nsplit) {
  if (dtype == ESP_BF16 && hd == 128) {   // ring layout: whole column tiles of 32
    const RingGeometry g = ring_geometry(rows_per_seq * (hq / hkv));
    return (size_t)batch * hkv * g.q_tiles * g.ct_wg * nsplit * (32 * (hd + 2));
  }
  return (size_t)batch * rows_per_seq * hq * nsplit * (hd + 2);
}

hipError_t launch_attn(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int layer, int hq, int hkv,
                       int hd, const void* q, float* partials, const AttnPlan& p) {
  const int M = b.batch * b.rows_per_seq;
  float* part_o = partials;
  float* part_ml = partials + (size_t)M * hq * p.nsplit * hd;
  if (dtype == ESP_BF16 && hd == 128) {
    const RingGeometry g = ring_geometry(b.rows_per_seq * (hq / hkv));
    part_ml = partials + (size_t)b.batch * hkv * g.q_tiles * g.ct_wg * p.nsplit * (32 * hd);
    const int total_wg = g.q_tiles * hkv * b.batch * p.nsplit;
    const hipError_t attr = attn_prepare();
    if (attr != hipSuccess) return attr;
    const dim3 grid(((total_wg + 7) / 8) * 8), block(64 * g.waves);
    if (g.waves >= 8)
      hipLaunchKernelGGL(k_attn_ring<4>, grid, block, RING_LDS_BYTES, st, b, kv, layer, hq, hkv, (const bf16_t*)q, part_o,
                         part_ml, p.nsplit, p.tiles_per_split, g.q_tiles, g.ct_wg, g.n_full);
    else
      hipLaunchKernelGGL(k_attn_ring<8>, grid, block, RING_LDS_BYTES, st, b, kv, layer, hq, hkv, (const bf16_t*)q, part_o,
                         part_ml, p.nsplit, p.tiles_per_split, g.q_tiles, g.ct_wg, g.n_full);
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

hipError_t launch_attn_merge(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int hq, int hkv, int hd,
                             const float* partials, const AttnPlan& p, void* out) {
  if (dtype == ESP_BF16 && hd == 128) {
    const RingGeometry g = ring_geometry(b.rows_per_seq * (hq / hkv));
    const int n_ct = g.q_tiles * g.ct_wg;
    const float* part_o = partials;
    const float* part_ml = partials + (size_t)b.batch * hkv * n_ct * p.nsplit * (32 * hd);
    const dim3 grid(b.batch * hkv * n_ct * 4);
    if (p.nsplit <= 64)
      hipLaunchKernelGGL(k_attn_merge_ring<64>, grid, dim3(256), 0, st, b, kv, hq, hkv, part_o, part_ml, p.nsplit, n_ct,
                         (bf16_t*)out);
    else
      return hipErrorInvalidValue;
    return hipGetLastError();
  }
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
