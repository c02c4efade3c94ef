// Fused vocabulary softmax + Top-K' of the mask-row logits (paper Sec. 2 Eq. 2, Sec. 3.3).
//
// Each logit row is read exactly once, by independent wavefronts and without a barrier.
// Pass 1 (k_topk_stream): a wave streams one segment of one row in blocks of 2048 logits
// (32 per lane, float4 loads, the next block in flight while the current one is reduced).
//   * softmax statistics stay lane-local (running maximum and rescaled sum of exponentials) and
//     are combined across the wave once, at the end of the segment;
//   * the K' best (value desc, id asc) live in a list spread over the lanes (lane j holds the
//     j-th best).  A block is only looked at when its maximum reaches the current K'-th value,
//     which after the first block is rare (about K' ln(n/K') times per n logits), so the common
//     path per logit is one max, one fma, one exp and one add.  The first block is filtered by the
//     K'-th largest of its 64 lane maxima (at least K' logits reach that bound), which keeps the
//     warm-up to a few insertions.
// Pass 2 (k_topk_merge): one wave per row merges the segment statistics (online-softmax rule) and
// the segments' sorted lists (at most 64 segments, one per lane: K' rounds of a wave-wide best-head
// search); p = exp(v - max) / sum in fp32.
#include <algorithm>
#include <mutex>

#include "esp_internal.h"

namespace {

constexpr int BLOCK = 2048;            // logits per wave and iteration
constexpr int PER_LANE = BLOCK / 64;
constexpr float LOG2E_F = 1.4426950408889634f;

__device__ __forceinline__ bool better(float av, int ai, float bv, int bi) {
  return av > bv || (av == bv && ai < bi);
}
__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// The K' best so far, lane j < kp holding the j-th; lanes >= kp hold (-inf, INT_MAX).
struct LaneList {
  float v;
  int id;
  float last_v;   // entry kp-1 (wave-uniform)
  int last_id;
};
__device__ __forceinline__ void list_init(LaneList& L) {
  L.v = -INFINITY; L.id = 0x7fffffff; L.last_v = -INFINITY; L.last_id = 0x7fffffff;
}
// insert (v, id), known to be better than the last entry; v, id wave-uniform
__device__ __forceinline__ void list_insert(LaneList& L, float v, int id, int kp, int lane) {
  const bool mine_better = lane < kp && better(L.v, L.id, v, id);
  const int pos = __popcll(__builtin_amdgcn_ballot_w64(mine_better));   // the better entries form a prefix
  const float up_v = __shfl_up(L.v, 1, 64);
  const int up_i = __shfl_up(L.id, 1, 64);
  if (lane < kp) {
    if (lane == pos) { L.v = v; L.id = id; }
    else if (lane > pos) { L.v = up_v; L.id = up_i; }
  }
  L.last_v = readlane_f(L.v, kp - 1);
  L.last_id = __builtin_amdgcn_readlane(L.id, kp - 1);
}

// kp-th largest of the 64 lane values (bitonic sort across the wave, descending); kp <= 64
__device__ __forceinline__ float kth_largest_lane(float x, int kp, int lane) {
#pragma unroll
  for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      const float o = __shfl_xor(x, j, 64);
      const bool desc = (lane & k) == 0;            // direction of this lane's subsequence
      const bool low = (lane & j) == 0;             // lower index of the pair
      const float hi = fmaxf(x, o), lo = fminf(x, o);
      x = (desc == low) ? hi : lo;
    }
  }
  return readlane_f(x, kp - 1);
}

// Offer the values of one register slot (one per lane) to the list: every lane whose value
// reaches the bound is examined in turn (wave-uniform loop over the ballot).
__device__ __forceinline__ void offer(LaneList& L, float v, int my_id, float& bound, float floor_bound, int kp,
                                      int lane) {
  unsigned long long mask = __builtin_amdgcn_ballot_w64(v >= bound);
  while (mask) {
    const int l = __builtin_ctzll(mask);
    mask &= mask - 1;
    const float cv = readlane_f(v, l);
    const int cid = __builtin_amdgcn_readlane(my_id, l);
    if (better(cv, cid, L.last_v, L.last_id)) {
      list_insert(L, cv, cid, kp, lane);
      bound = fmaxf(floor_bound, L.last_v);
      mask &= __builtin_amdgcn_ballot_w64(v >= bound);
    }
  }
}

// record per (row, segment): [max, sum, v_0..v_{kp-1}, id_0..id_{kp-1}] as 2 + 2*kp words
__global__ __launch_bounds__(256) void k_topk_stream(const float* __restrict__ logits, int rows, int vocab, int kp,
                                                     int nseg, int seg_len, float* __restrict__ seg_rec,
                                                     const int32_t* __restrict__ row_map) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= rows * nseg) return;
  const int row = item / nseg, seg = item % nseg;
  const int start = seg * seg_len, end = min(vocab, start + seg_len);
  const float* p = logits + (size_t)(row_map ? max(row_map[row], 0) : row) * vocab;
  const bool vec4 = (vocab & 3) == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0;
  const int nblocks = (max(end - start, 0) + BLOCK - 1) / BLOCK;

  // element e of float4 i of the lane sits at block_base + i*256 + lane*4 + e
  float nxt[PER_LANE], cur[PER_LANE];
  auto load_block = [&](int b, float (&dst)[PER_LANE]) {
    const int base = start + b * BLOCK + lane * 4;
    if (vec4 && start + (b + 1) * BLOCK <= end) {
#pragma unroll
      for (int i = 0; i < PER_LANE / 4; ++i) {
        const f32x4_t q = *reinterpret_cast<const f32x4_t*>(p + base + i * 256);
        dst[4 * i] = q[0]; dst[4 * i + 1] = q[1]; dst[4 * i + 2] = q[2]; dst[4 * i + 3] = q[3];
      }
    } else {
#pragma unroll
      for (int i = 0; i < PER_LANE; ++i) {
        const int idx = base + (i >> 2) * 256 + (i & 3);
        dst[i] = idx < end ? p[idx] : -INFINITY;
      }
    }
  };

  LaneList L;
  list_init(L);
  float m = -INFINITY, s = 0.f;       // lane-local running maximum and sum of 2^((v - m) log2 e)
  float floor_bound = -INFINITY, bound = -INFINITY;
  if (nblocks > 0) load_block(0, nxt);
  for (int b = 0; b < nblocks; ++b) {
#pragma unroll
    for (int i = 0; i < PER_LANE; ++i) cur[i] = nxt[i];
    if (b + 1 < nblocks) load_block(b + 1, nxt);
    float bmax = cur[0];
#pragma unroll
    for (int i = 1; i < PER_LANE; ++i) bmax = fmaxf(bmax, cur[i]);
    const float m_new = fmaxf(m, bmax);
    if (m_new > -INFINITY) {
      const float mb = m_new * LOG2E_F;
      float acc = s * __builtin_amdgcn_exp2f(m * LOG2E_F - mb);   // m = -inf: 0
#pragma unroll
      for (int i = 0; i < PER_LANE; ++i) acc += __builtin_amdgcn_exp2f(fmaf(cur[i], LOG2E_F, -mb));
      s = acc;
      m = m_new;
    }
    if (b == 0) {
      floor_bound = kth_largest_lane(bmax, kp, lane);
      bound = floor_bound;
    }
    if (__builtin_amdgcn_ballot_w64(bmax >= bound) != 0ull) {
      const int base = start + b * BLOCK + lane * 4;
#pragma unroll
      for (int i = 0; i < PER_LANE; ++i) offer(L, cur[i], base + (i >> 2) * 256 + (i & 3), bound, floor_bound, kp, lane);
    }
  }
  // wave-wide statistics in the natural-exponent convention: sum of exp(v - max)
  const float wm = wave_max(m);
  const float contrib = m > -INFINITY ? s * __builtin_amdgcn_exp2f((m - wm) * LOG2E_F) : 0.f;
  const float ws = wave_sum(contrib);
  float* out = seg_rec + ((size_t)row * nseg + seg) * (2 + 2 * kp);
  if (lane == 0) { out[0] = wm; out[1] = ws; }
  if (lane < kp) {
    out[2 + lane] = L.v;
    reinterpret_cast<int*>(out)[2 + kp + lane] = L.id;
  }
}

// one wave per row: the segments' lists are sorted, so lane c walks segment c's list and the wave
// takes the best head (value desc, id asc) K' times -- a 64-way merge of sorted lists
__global__ __launch_bounds__(256) void k_topk_merge(const float* __restrict__ seg_rec, int rows, int kp, int nseg,
                                                    int32_t* __restrict__ ids, float* __restrict__ probs) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int stride = 2 + 2 * kp;
  const float* e = seg_rec + ((size_t)row * nseg + lane) * stride;     // this lane's segment (nseg <= 64)
  const bool have = lane < nseg;
  const float smax = have ? e[0] : -INFINITY;
  const float gmax = wave_max(smax);
  const float tot = wave_sum(have && smax > -INFINITY ? e[1] * expf(smax - gmax) : 0.f);
  int pos = 0;                                                          // next unread entry of the list
  float hv = have ? e[2] : -INFINITY;
  int hi = have ? reinterpret_cast<const int*>(e)[2 + kp] : 0x7fffffff;
  if (hv == -INFINITY) hi = 0x7fffffff;                                 // empty slot: never wins
  float out_v = -INFINITY;
  int out_i = 0x7fffffff;
  for (int j = 0; j < kp; ++j) {
    float bv = hv;
    int bi = hi;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (lane == j) { out_v = bv; out_i = bi; }
    if (hi == bi && bi != 0x7fffffff) {                                 // ids are unique: exactly one lane advances
      ++pos;
      hv = pos < kp ? e[2 + pos] : -INFINITY;
      hi = pos < kp ? reinterpret_cast<const int*>(e)[2 + kp + pos] : 0x7fffffff;
      if (hv == -INFINITY) hi = 0x7fffffff;
    }
  }
  if (lane < kp) {
    const bool any = out_i != 0x7fffffff;
    ids[(size_t)row * kp + lane] = any ? out_i : -1;
    probs[(size_t)row * kp + lane] = any ? expf(out_v - gmax) / tot : 0.f;
  }
}

// segments per row: enough independent waves to fill the chip (about 8 per CU), each at least one
// block long
int topk_segments(int rows, int vocab, int* seg_len) {
  const int max_seg = std::min(64, (vocab + BLOCK - 1) / BLOCK);   // the merge gives each segment a lane
  int nseg = std::max(1, std::min(max_seg, (2048 + rows - 1) / rows));
  int len = ((vocab + nseg - 1) / nseg + BLOCK - 1) / BLOCK * BLOCK;
  nseg = (vocab + len - 1) / len;
  *seg_len = len;
  return nseg;
}

// ---- entry point for callers that cannot allocate ---------------------------------------------
// Per-(row, segment) statistics and candidate lists of the two-pass Top-K' in a file-scope device
// array instead of a caller workspace.  Every GPU the library runs on holds its own copy of the
// array (at its own address) until the process ends; the host-side name is only a handle for
// hipGetSymbolAddress, whose result (per device) is what the kernels receive.
constexpr int STATIC_MAX_ROWS = 128;
constexpr size_t STATIC_SCRATCH_FLOATS = (size_t)STATIC_MAX_ROWS * 64 * (2 + 2 * ESP_MAX_TOPK);   // 2.06 MiB
static __device__ __align__(256) __attribute__((used)) float scratch[STATIC_SCRATCH_FLOATS];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static float* g_scratch_ptr[MAX_DEVICES] = {};   // device address of `scratch` on each device, 0 = not looked up yet

// device address of the array on the current device (looked up once per device)
static hipError_t static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" esp_status esp_softmax_topk_static(void* stream, const float* logits, int32_t rows, int32_t vocab,
                                              int32_t Kp, int32_t* ids, float* probs) {
  if (!logits || !ids || !probs) return ESP_EINVAL;
  if (rows < 1 || vocab < 1 || Kp < 1 || Kp > ESP_MAX_TOPK || Kp > vocab) return ESP_EINVAL;
  if (softmax_topk_scratch_floats(rows, vocab, Kp) > STATIC_SCRATCH_FLOATS) return ESP_ECAPACITY;
  float* ws = nullptr;
  if (static_scratch(&ws) != hipSuccess) return ESP_EDEVICE;
  // every (row, segment) record the merge pass reads is written by the stream pass of the same
  // call, so nothing of an earlier call's contents has to be cleared
  if (launch_softmax_topk((hipStream_t)stream, logits, rows, vocab, Kp, ids, probs, ws, nullptr) != hipSuccess)
    return ESP_EDEVICE;
  return ESP_OK;
}

size_t softmax_topk_scratch_floats(int rows, int vocab, int kp) {
  int max_seg = std::min(64, (vocab + BLOCK - 1) / BLOCK);   // upper bound of the segment count for any row count
  return (size_t)rows * max_seg * (2 + 2 * kp);
}

hipError_t launch_softmax_topk(hipStream_t st, const float* logits, int rows, int vocab, int kp, int32_t* ids,
                               float* probs, float* ws, const int32_t* row_map) {
  if (rows <= 0) return hipSuccess;
  int seg_len = 0;
  const int nseg = topk_segments(rows, vocab, &seg_len);
  const int items = rows * nseg;
  hipLaunchKernelGGL(k_topk_stream, dim3((items + 3) / 4), dim3(256), 0, st, logits, rows, vocab, kp, nseg, seg_len,
                     ws, row_map);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_topk_merge, dim3((rows + 3) / 4), dim3(256), 0, st, ws, rows, kp, nseg, ids, probs);
  return hipGetLastError();
}
