// Internal declarations shared by the HIP sources of libesp_hip.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

#include "esp.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));   // 16 raw bytes in registers

#define ESP_WAVE 64

// ---- element conversion -----------------------------------------------------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- direct global -> LDS loads --------------------------------------------------------------
// One 16-byte piece per lane from global memory straight into LDS (no register hop): the lane
// supplies its own global address, the wave's 64 pieces land at lds_addr + 16 * lane.  Issued as
// text so that the compiler's wait-count bookkeeping knows nothing of it: the LDS rings of the GEMM
// and attention kernels count their own loads (they retire in order) and would otherwise be
// drained before every LDS read.
// M0 (the LDS base of the transfer) is put back to what it held before, so the statement leaves no
// register changed that the compiler might rely on.
__device__ __forceinline__ void load_to_lds16(const void* g, uint32_t lds_addr) {
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "s"(lds_addr), "v"(g)
               : "memory");
}
// The same with a wave-uniform base address (scalar registers) plus a per-lane byte offset and a
// constant offset IMM, which the hardware adds to the global address and to the LDS address alike
// (piece j of a run: IMM = j KB, lds_addr the address of piece 0): one vector register for any
// number of pieces.
template <int IMM>
__device__ __forceinline__ void load_to_lds16_sbase(const void* sbase, uint32_t lane_off, uint32_t lds_addr) {
  uint32_t keep;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3 offset:%4\n\ts_mov_b32 m0, %0"
      : "=&s"(keep)
      : "s"(lds_addr), "v"(lane_off), "s"(sbase), "n"(IMM)
      : "memory");
}
template <int N_YOUNGER>
__device__ __forceinline__ void wait_loads_but() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_YOUNGER) : "memory");
}

// ---- sample matching (temperature 1): counter-based Gumbel noise ---------------------------------
// u in (0,1) from a 32-bit multiply-xorshift mix (MurmurHash3 finaliser family) of (seed, position,
// token id), top 23 bits centred in their cell (exact in fp32); g = -ln(-ln u) is standard Gumbel, and
// arg-max over the vocabulary of logit + g is a draw from softmax(logits).  `position` is the absolute
// position of the token being drawn, so a draw does not depend on how its position is reached.
__device__ __forceinline__ float gumbel_noise(uint32_t seed, uint32_t position, uint32_t id) {
  uint32_t x = id * 0x9E3779B1u + position * 0x85EBCA77u + seed * 0xC2B2AE3Du;
  x ^= x >> 16; x *= 0x85EBCA6Bu; x ^= x >> 13; x *= 0xC2B2AE35u; x ^= x >> 16;
  const float u = ((float)(x >> 9) + 0.5f) * (1.0f / 8388608.0f);
  return -logf(-logf(u));
}

// ---- KV cache addressing (see esp_kv in esp.h) --------------------------------------------
// Per (layer, kv head) plane of capacity*hd elements, in blocks of 32 slots stored in the order
// the matrix cores consume them (v_mfma_f32_32x32x16 A operands, 64 lanes x 8 elements each):
//   K block: [hd/16 k-steps][64 lanes][8]   lane (slot%32, half) holds features 16*step + 8*half + 0..7
//            (A operand of S^T = K Q^T: row = key, contraction over features)
//   V block: [hd/32 feature blocks][2 key-steps][64 lanes][8]   lane (feature%32, half), element j
//            holds key 16*step + 8*(j/4) + 4*half + j%4 -- the order in which the S^T accumulator
//            registers of a lane half line up as B operand of O^T = V^T P^T
// so a tile of keys is one contiguous run of bytes and every fragment is one 16-byte load per lane.
__host__ __device__ __forceinline__ size_t kv_plane(int layer, int kvh, int n_kv, int64_t cap, int hd) {
  return ((size_t)layer * n_kv + kvh) * (size_t)cap * hd;
}
__host__ __device__ __forceinline__ size_t k_off(int64_t slot, int d, int hd) {
  return (size_t)(slot >> 5) * hd * 32 + (size_t)((((d >> 4) * 64 + ((d >> 3) & 1) * 32 + (int)(slot & 31)) << 3) + (d & 7));
}
__host__ __device__ __forceinline__ size_t v_off(int64_t slot, int d, int hd) {
  const int key = (int)(slot & 31), u = key >> 4, half = (key >> 2) & 1, j = ((key >> 3) & 1) * 4 + (key & 3);
  return (size_t)(slot >> 5) * hd * 32 + (size_t)(((((d >> 5) * 2 + u) * 64 + half * 32 + (d & 31)) << 3) + j);
}

// ---- GEMM -----------------------------------------------------------------------------------
struct GemmPlan {
  int splits;        // split-K factor; a function of (N, K) and of the tile class (<=128 rows or more)
  int mt;            // 32-row MFMA tiles per workgroup
  int nb;            // 32-column blocks per wave
  int m_tiles;       // workgroup tiles along M
  int n_tiles;       // workgroup tiles along N
  int wm;            // wave groups along M inside a workgroup (1: 256 threads, 2: 512 threads)
};
GemmPlan gemm_plan(int dtype, int M, int N, int K);
inline size_t gemm_out_elems(const GemmPlan& p, int M, int N) { return (size_t)p.splits * M * N; }
// out: fp32 [splits][M][N].  a_rows (device, may be null): physical row of A for logical row m.
// w_packed: W is in the streaming layout written by launch_pack_weight (bf16 only).
hipError_t launch_gemm(hipStream_t st, int dtype, const void* A, const int32_t* a_rows, const void* W,
                       float* out, int M, int N, int K, const GemmPlan& p, bool w_packed, int a_ld = 0);
// a_ld == 0: A is row-major [rows][K]; a_ld > 0 (bf16 only): A is chunk-major [K/64][a_ld][64]
hipError_t launch_pack_weight(hipStream_t st, const void* src, void* dst, int N, int K);
// one-time kernel attributes of the GEMM kernels (dynamic LDS limits); call before the first launch
hipError_t gemm_prepare();
hipError_t launch_gemm_swiglu(hipStream_t st, const void* A, const void* W, void* act, int M, int ff, int K);
// LM head with the arg-max taken in the GEMM epilogue (bf16, packed weights, <= 128 rows, one split)
bool gemm_argmax_supported(int dtype, int M, int N, int K, bool with_logits);
size_t gemm_argmax_scratch_floats(int M, int N);
// logits_out == NULL: arg-max of each of the M rows (out[out_index[m]]), logits never written.
// logits_out != NULL: also writes the fp32 logits [M][N]; arg-max only for the n_arg rows arg_rows[i].
hipError_t launch_gemm_argmax(hipStream_t st, const void* A, const int32_t* a_rows, const void* W, int M, int N,
                              int K, float* scratch, int32_t* out, const int32_t* out_index, int a_ld,
                              float* logits_out, const int32_t* arg_rows, int n_arg,
                              const int32_t* draw_pos = nullptr, uint32_t seed = 0);   // draw_pos: per GEMM row

// ---- elementwise / glue (esp_elementwise.hip) ----------------------------------------------
struct BlockDev {   // device-side view of esp_block + esp_kv scalars, passed by value
  int batch, rows_per_seq, k_masks, layout, anc_words;
  const int32_t *n_rows, *n_nodes, *tok, *parent, *depth, *mask_j, *attach;
  const uint64_t* anc;
};
struct KvDev {
  void *k, *v;
  int32_t* len;
  const int32_t *base, *seq_cap;
  int64_t capacity;
  int len_bound;
};

hipError_t launch_embed(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, const void* embed,
                        const void* mask_embed, float* h, int d, int vocab, float* rope_tab, int hd,
                        float theta, int32_t* status, size_t mask_seq_stride);
hipError_t launch_residual_norm(hipStream_t st, int dtype, float* h, const float* part, int splits, int M,
                                int d, const void* gain, float eps, void* xn_out);
hipError_t launch_qkv_post(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int layer,
                           const float* part, int splits, int M, int hq, int hkv, int hd, int qk_norm,
                           const void* qg, const void* kg, float eps, const float* rope_tab, void* q_out);
hipError_t launch_swiglu(hipStream_t st, int dtype, const float* part, int splits, int M, int dff, void* act);
// draw_pos (nullable): sample instead of arg-max -- entry m draws position draw_pos[m] with `seed`
hipError_t launch_argmax(hipStream_t st, const float* logits, size_t row_stride, const int32_t* row_map,
                         int n_rows_out, int vocab, int32_t* out, const int32_t* out_index,
                         const int32_t* draw_pos = nullptr, uint32_t seed = 0);
// pos_list (nullable): position of the token that follows node-list entry m (len + depth + 1)
hipError_t launch_node_rows(hipStream_t st, const BlockDev& b, int max_nodes, int32_t* a_rows, int32_t* out_rows,
                            const int32_t* kv_len = nullptr, int32_t* pos_list = nullptr);
// pos_rows[row] = len[seq] + depth[row] + 1 for every block row
hipError_t launch_row_positions(hipStream_t st, const BlockDev& b, const int32_t* kv_len, int32_t* pos_rows);
hipError_t launch_kv_copy(hipStream_t st, int dtype, const KvDev& kv, int layer, int n_kv, int hd,
                          int seq_base, int first_slot, int n_slots, void* k_rows, void* v_rows, int to_cache);
hipError_t launch_mask_mean(hipStream_t st, int dtype, const void* embed, const int32_t* tokens, int n, int k,
                            int d, int vocab, void* mask_embed);
hipError_t launch_mask_last_k(hipStream_t st, int dtype, const void* embed, const int32_t* tokens, int n, int k,
                              int d, int vocab, void* mask_embed);
size_t mask_gaussian_scratch_floats(int d);
hipError_t launch_mask_gaussian(hipStream_t st, int dtype, const void* embed, int vocab, int d, const float* z,
                                float shift, int k, float* scratch, size_t scratch_floats, void* mask_embed);
hipError_t launch_mask_ema(hipStream_t st, int dtype, const void* embed, const int32_t* n_emit,
                           const int32_t* emit_tok, float lambda, int k, int d, int vocab, void* mask_embed, int n_seq);

// ---- attention (esp_attn.hip) ------------------------------------------------------------------
struct AttnPlan { int nsplit; int tiles_per_split; };
AttnPlan attn_plan(int batch, int rows_per_seq, int hq, int hkv, int len_bound);
hipError_t attn_prepare();   // one-time kernel attributes (dynamic LDS limit)
size_t attn_partial_floats(int dtype, int batch, int rows_per_seq, int hq, int hkv, int hd, int nsplit);
hipError_t launch_attn(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int layer, int hq,
                       int hkv, int hd, const void* q, float* partials, const AttnPlan& p);
hipError_t launch_attn_merge(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv, int hq, int hkv, int hd,
                             const float* partials, const AttnPlan& p, void* out);

// ---- softmax + top-k (esp_topk.hip) -----------------------------------------------------------
size_t softmax_topk_scratch_floats(int rows, int vocab, int kp);
// row_map (nullable): logits row of output row r is row_map[r] (negative: 0)
hipError_t launch_softmax_topk(hipStream_t st, const float* logits, int rows, int vocab, int kp, int32_t* ids,
                               float* probs, float* scratch, const int32_t* row_map = nullptr);

// ---- tree logic (esp_tree.hip) -------------------------------------------------------------------
hipError_t launch_block_from_tree(hipStream_t st, int batch, int rows_per_seq, int k, int layout, int anc_words,
                                  int32_t* n_rows, const int32_t* n_nodes, int32_t* tok, int32_t* parent,
                                  int32_t* depth, int32_t* mask_j, int32_t* attach, uint64_t* anc,
                                  int32_t* status);
hipError_t launch_verify_accept(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv,
                                const int32_t* node_argmax, int n_layers, int n_kv, int hd, int32_t* n_emit,
                                int32_t* emit_tok, int32_t* accepted_row, int32_t* star_row, int32_t* status);
hipError_t launch_mask_rows(hipStream_t st, const BlockDev& b, const int32_t* star_row, const int32_t* n_emit,
                            int32_t* a_rows, int32_t* n_lists);
hipError_t launch_build_tree(hipStream_t st, const esp_tree_params& p, int batch, const int32_t* topk_id,
                             const float* topk_p, int kp, const int32_t* n_lists, const int32_t* n_emit,
                             const int32_t* emit_tok, int rows_per_seq, int anc_words, int32_t* n_rows,
                             int32_t* n_nodes, int32_t* tok, int32_t* parent, int32_t* depth, int32_t* mask_j,
                             int32_t* attach, uint64_t* anc, int32_t* status, bool reuse);

// Events a profiling scope hands to the next bf16 GEMM launch: the launch attaches them to the kernel
// itself (hipExtLaunchKernelGGL), so they carry the kernel's own begin and end time stamps and not the
// time of two extra event commands around it.
struct LaunchEvents { hipEvent_t start = nullptr, stop = nullptr; };
extern thread_local LaunchEvents g_launch_events;

// ---- context --------------------------------------------------------------------------------------
struct esp_ctx {
  esp_model_desc m;
  const void *embed, *lm_head, *final_norm;
  std::vector<const void*> wqkv, wo, wgu, wdown, norm_attn, norm_mlp, q_norm, k_norm;
  int max_batch, max_rows;
  int64_t max_kv_len;
  hipStream_t stream;
  char* ws;
  size_t ws_bytes;
  // workspace partition
  float* h;          // [Mmax][d] fp32 residual stream
  void* xn;          // T [Mmax][d]
  void* q;           // T [Mmax][hq*hd]
  void* attn_out;    // T [Mmax][hq*hd]
  void* act;         // T [Mmax][d_ff]
  float* gemm_out;   // fp32 split-K partials of the largest layer GEMM
  float* attn_part;  // attention split partials
  // logits of all block rows left in `logits` by the last esp_tree_forward (bf16, <= 128 rows), for
  // esp_mask_topk on the same hidden states: the hidden buffer they came from and the row count
  int sample_on = 0;            // sample matching instead of greedy verification
  uint32_t sample_seed = 0;
  int32_t *idx_c, *idx_d;       // draw positions per block row / per node-list entry
  const void* lm_cache_hidden = nullptr;
  int lm_cache_rows = 0;
  // blocks that hold the rows of a fixed tree built with these parameters (esp_build_prune_tree
  // then only rewrites their tokens): identity = address of the block's token array
  bool mask_per_seq = false;    // mask vectors are [batch, k, d] (esp_set_mask_batch)
  struct StaticTreeSlot { const void* tok = nullptr; uint64_t sig = 0; };
  StaticTreeSlot static_trees[4];
  float* rope_tab;   // [Mmax][hd/2][2] cos, sin
  float* logits;     // fp32 [logits_rows][vocab]
  float* topk_scratch;
  int32_t* idx_a;    // [Mmax] gather rows
  int32_t* idx_b;    // [Mmax]
  int32_t* status;   // device status word
  size_t gemm_out_floats, attn_part_floats, logits_rows;
  // optional launch-site timing with HIP events (esp_profile_enable / esp_profile_read)
  struct ProfSpan { int site; hipEvent_t start, stop; };
  uint32_t prof_mask = 0;
  std::vector<ProfSpan> prof_open;
  std::vector<hipEvent_t> prof_pool;
  double prof_ms[ESP_SITE_COUNT] = {};
  int64_t prof_n[ESP_SITE_COUNT] = {};
};
