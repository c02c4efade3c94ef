// Fused vocabulary softmax + Top-K' of the mask-row logits (paper Sec. 2 Eq. 2, Sec. 3.3).
//
// Each logit row is read exactly once.  Pass 1: a workgroup takes a chunk of 2048 logits of one
// row into registers, reduces the chunk maximum and sum of exponentials (wavefront shuffles, then
// LDS across the four waves) and extracts the chunk's K' largest (value desc, id asc) by K' rounds
// of block arg-max.  Pass 2: one workgroup per row merges the chunk statistics (online-softmax
// rule) and selects the K' best of the chunk winners from LDS; p = exp(v - max) / sum in fp32.
#include "esp_internal.h"

namespace {

constexpr int CHUNK = 2048;
constexpr int PER_THREAD = CHUNK / 256;

struct Best {
  float v;
  int id;
};
__device__ __forceinline__ bool better(float av, int ai, float bv, int bi) {
  return av > bv || (av == bv && ai < bi);
}
__device__ __forceinline__ Best wave_best(Best b) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(b.v, o, 64);
    int oi = __shfl_xor(b.id, o, 64);
    if (better(ov, oi, b.v, b.id)) { b.v = ov; b.id = oi; }
  }
  return b;
}
// all threads get the block-wide best; sv/si are 4-entry LDS arrays
__device__ __forceinline__ Best block_best(Best b, float* sv, int* si) {
  b = wave_best(b);
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = b.v; si[threadIdx.x >> 6] = b.id; }
  __syncthreads();
  Best r = {sv[0], si[0]};
#pragma unroll
  for (int w = 1; w < 4; ++w)
    if (better(sv[w], si[w], r.v, r.id)) { r.v = sv[w]; r.id = si[w]; }
  __syncthreads();
  return r;
}

// scratch per (row, chunk): [max, sum, v_0..v_{kp-1}, id_0..id_{kp-1}] as 2 + 2*kp words
__global__ __launch_bounds__(256) void k_topk_chunks(const float* __restrict__ logits, int vocab, int kp,
                                                     int nchunks, float* __restrict__ scratch) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int row = blockIdx.y, chunk = blockIdx.x, tid = threadIdx.x;
  const float* p = logits + (size_t)row * vocab;
  const int c0 = chunk * CHUNK;
  float v[PER_THREAD];
  float lmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) {
    int idx = c0 + i * 256 + tid;
    v[i] = idx < vocab ? p[idx] : -INFINITY;
    lmax = fmaxf(lmax, v[i]);
  }
  float cmax = wave_max(lmax);
  if ((tid & 63) == 0) sv[tid >> 6] = cmax;
  __syncthreads();
  cmax = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
  __syncthreads();
  float lsum = 0.f;
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i) lsum += v[i] == -INFINITY ? 0.f : expf(v[i] - cmax);
  float csum = wave_sum(lsum);
  if ((tid & 63) == 0) sv[tid >> 6] = csum;
  __syncthreads();
  csum = (sv[0] + sv[1]) + (sv[2] + sv[3]);
  __syncthreads();
  float* out = scratch + ((size_t)row * nchunks + chunk) * (2 + 2 * kp);
  if (tid == 0) { out[0] = cmax; out[1] = csum; }
  for (int j = 0; j < kp; ++j) {
    Best mine = {-INFINITY, 0x7fffffff};
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      int idx = c0 + i * 256 + tid;
      if (better(v[i], idx, mine.v, mine.id) && v[i] != -INFINITY) { mine.v = v[i]; mine.id = idx; }
    }
    Best win = block_best(mine, sv, si);
    if (tid == 0) {
      out[2 + j] = win.v;
      reinterpret_cast<int*>(out)[2 + kp + j] = win.id;
    }
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i)
      if (c0 + i * 256 + tid == win.id) v[i] = -INFINITY;
  }
}

__global__ __launch_bounds__(256) void k_topk_merge(const float* __restrict__ scratch, int kp, int nchunks,
                                                    int32_t* __restrict__ ids, float* __restrict__ probs) {
  extern __shared__ float cand[];     // [nchunks*kp] values then [nchunks*kp] ids
  __shared__ float sv[4];
  __shared__ int si[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int ncand = nchunks * kp;
  float* cv = cand;
  int* ci = reinterpret_cast<int*>(cand + ncand);
  const float* base = scratch + (size_t)row * nchunks * (2 + 2 * kp);
  float lmax = -INFINITY;
  for (int c = tid; c < nchunks; c += 256) lmax = fmaxf(lmax, base[(size_t)c * (2 + 2 * kp)]);
  float gmax = wave_max(lmax);
  if ((tid & 63) == 0) sv[tid >> 6] = gmax;
  __syncthreads();
  gmax = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
  __syncthreads();
  float lsum = 0.f;
  for (int c = tid; c < nchunks; c += 256) {
    const float* e = base + (size_t)c * (2 + 2 * kp);
    lsum += e[1] * expf(e[0] - gmax);
  }
  float tot = wave_sum(lsum);
  if ((tid & 63) == 0) sv[tid >> 6] = tot;
  __syncthreads();
  tot = (sv[0] + sv[1]) + (sv[2] + sv[3]);
  __syncthreads();
  for (int i = tid; i < ncand; i += 256) {
    const float* e = base + (size_t)(i / kp) * (2 + 2 * kp);
    cv[i] = e[2 + i % kp];
    ci[i] = reinterpret_cast<const int*>(e)[2 + kp + i % kp];
  }
  __syncthreads();
  for (int j = 0; j < kp; ++j) {
    Best mine = {-INFINITY, 0x7fffffff};
    for (int i = tid; i < ncand; i += 256)
      if (cv[i] != -INFINITY && better(cv[i], ci[i], mine.v, mine.id)) { mine.v = cv[i]; mine.id = ci[i]; }
    Best win = block_best(mine, sv, si);
    if (tid == 0) {
      bool any = win.id != 0x7fffffff;
      ids[(size_t)row * kp + j] = any ? win.id : -1;
      probs[(size_t)row * kp + j] = any ? expf(win.v - gmax) / tot : 0.f;
    }
    for (int i = tid; i < ncand; i += 256)
      if (ci[i] == win.id) cv[i] = -INFINITY;
    __syncthreads();
  }
}

}  // namespace

size_t softmax_topk_scratch_floats(int rows, int vocab, int kp) {
  int nchunks = (vocab + CHUNK - 1) / CHUNK;
  return (size_t)rows * nchunks * (2 + 2 * kp);
}

hipError_t launch_softmax_topk(hipStream_t st, const float* logits, int rows, int vocab, int kp, int32_t* ids,
                               float* probs, float* scratch) {
  if (rows <= 0) return hipSuccess;
  int nchunks = (vocab + CHUNK - 1) / CHUNK;
  hipLaunchKernelGGL(k_topk_chunks, dim3(nchunks, rows), dim3(256), 0, st, logits, vocab, kp, nchunks, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  size_t lds = (size_t)nchunks * kp * 8;
  hipLaunchKernelGGL(k_topk_merge, dim3(rows), dim3(256), lds, st, scratch, kp, nchunks, ids, probs);
  return hipGetLastError();
}
