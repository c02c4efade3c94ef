// Dense projections of the decoder: out[s][M][N] (fp32 partial sums over split s) = A[M,K] * W[N,K]^T.
//
// bf16 path (the 8B-class workloads): M is the number of block rows (tens to hundreds) while W is
// hundreds of MB per layer, so the kernel is a weight streamer.
//  * Weights live in HBM in a streaming layout (k_pack_weight): the 32-row x 64-k tile of a wave and
//    K-chunk is stored as [step][lane][8 values] = 4 KB contiguous in MFMA B-operand order, so every
//    wave-wide load covers 1 KB of consecutive addresses and the data goes HBM -> VGPR -> MFMA with no
//    LDS hop.  Tiles are ordered chunk-major ([chunk][row block]): at any moment the waves of the
//    whole grid, which advance through the chunks together, read one contiguous window of HBM.
//    Inside a chunk the k index is permuted identically for both operands (lane group g, step s
//    holds k = 32 g + 8 s + 0..7), which leaves the dot product unchanged.
//  * Large tiles (>= 8 MFMA tiles per wave; k_gemm_bf16_ring): both operands go global -> LDS
//    directly (global_load_lds_dwordx4, no register hop) into a ring of three chunk stages that
//    fills all but 4 KB of the CU's LDS.  Four computing waves (one per SIMD) only read fragments
//    and issue MFMAs; four loading waves (the second wave of each SIMD) issue the loads of chunk
//    c+2 while chunk c is computed.  Smaller tiles keep the operands in register rings:
//  * A register ring keeps D chunks of weights in flight per wave.  The activations of a chunk (L2
//    resident, shared by the four waves through LDS) ride in a ring of the same depth and are issued
//    together with the weights of the same chunk: loads retire in order, so waiting for the
//    activations of chunk c+1 leaves the D-2 younger chunks of the weight stream in flight.
//  * v_mfma_f32_32x32x16_bf16, fp32 accumulation; LDS fragment reads are double-buffered one MFMA
//    step ahead.
//  * Split-K (grid z): partial sums are reduced by the consumer in split order, so a result does
//    not depend on scheduling.  The split count is a function of (N, K) up to 128 rows; above, it
//    also depends on the number of row tiles (gemm_plan), so a row's low-order bits can differ
//    between a block of 320 rows and a block of 68.
//
// fp32 path (tiny configuration): plain LDS-tiled FMA kernel with bounds checks, row-major weights.
#include <algorithm>

#include <hip/hip_ext.h>

#include "esp_internal.h"

namespace {


constexpr int KC = 64;            // k per chunk
// silu(g) * u with the hardware exponential and reciprocal (about 1 ulp each; the result is
// rounded to bf16 next)
__device__ __forceinline__ float silu_mul(float g, float u) {
  return g * u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
}

constexpr int A_ROW_BYTES = 144;  // 128 B of bf16 + 16 B pad: conflict-free ds_read_b128 over 8 rows

// EPI: epilogue -- 0 fp32 tile out, 1 per-row arg-max over the workgroup's columns (pairs to out),
// 2 SwiGLU of interleaved gate/up column blocks to bf16, 3 fp32 tile to out and arg-max pairs to out2
// RING > 0 (packed weights only): both operands ride a ring of RING chunk stages in LDS, filled
// by load_to_lds16 two chunks ahead of their use; RING == 0: register rings of depth D.
template <int MT, int NB, int D, bool TILED, int WM, int EPI, int RING = 0>   // D even; WM wave groups along M
__device__ __forceinline__ void gemm_bf16_body(unsigned char* lds, const bf16_t* __restrict__ A,
                                               const int32_t* __restrict__ a_rows, const bf16_t* __restrict__ W,
                                               float* __restrict__ out, int M, int N, int K, int splits,
                                               int m_tiles, int n_tiles, int a_ld, float* __restrict__ out2,
                                               const int32_t* __restrict__ draw_pos, uint32_t seed) {
  // XCD-aware logical id: consecutive hardware ids go to different XCDs, so give each XCD a
  // contiguous range of tiles (tiles sharing weight rows then share an L2).
  const int total = m_tiles * n_tiles * splits;
  const int per_xcd = (total + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= total) return;
  const int mi = logical % m_tiles;
  const int ni = (logical / m_tiles) % n_tiles;
  const int z = logical / (m_tiles * n_tiles);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int lr = lane & 31, lg = lane >> 5;
  const int wn = wave & 3, wm = wave >> 2;       // column group, row group of this wave
  const int mt0 = mi * (WM * MT * 32);           // first row of the workgroup tile
  const int m0 = mt0 + wm * (MT * 32);           // first row of this wave
  const int n0 = ni * (128 * NB) + wn * (32 * NB);

  const int chunks = K / KC;
  const int cps = (chunks + splits - 1) / splits;
  const int c_begin = z * cps;
  const int c_end = min(chunks, c_begin + cps);

  f32x16_t acc[MT][NB];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if constexpr (RING > 0) {
    static_assert(TILED && WM == 1, "the ring path streams packed weights");
    // A stage holds chunk c of both operands, 1 KB per wave-load:
    //   activations [MT row tiles][32 rows][128 bytes], then weights [4 waves][NB column blocks]
    //   [4 steps] in MFMA fragment order (a linear copy of the packed layout).
    // An activation wave-load covers 8 rows of 128 bytes (8 lanes per row, so the global side stays
    // coalesced); within a row the eight 16-byte pieces are stored XOR-swizzled by the row index
    // (the lane fetches piece col ^ swz(row) for slot col), which makes the fragment reads -- lane
    // (r, g) wants piece 4 g + s of row r -- free of bank conflicts without padding.  Wave w brings
    // in the activation quarter-tiles w, w + 4, ... and its own weights.
    constexpr int A_STAGE = MT * 4096, STAGE = A_STAGE + 4 * NB * 4096;
    constexpr int LOADS = MT + 4 * NB;                    // per wave and chunk
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const bool loader = wave_u >= 4;                      // waves 4..7 only move data, for waves 0..3
    const int lw = wave_u & 3;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
    auto swz = [](int r) { return (r & 7) ^ ((r >> 3) & 1); };
    // Every load is "wave-uniform base in scalar registers + per-lane byte offset + constant": the
    // chunk index only moves the scalar base, so issuing a load costs no vector instruction besides
    // the load itself (address arithmetic in the vector unit would take issue slots from the MFMAs).
    uint32_t aoff[MT];                                    // byte offset of this lane's piece within a chunk's rows
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      const int pr = lw + 4 * j;                          // row tile pr / 4, rows 8 (pr % 4) .. + 7 of it
      const int rt = 8 * (pr & 3) + (lane >> 3);
      int m = min(mt0 + (pr >> 2) * 32 + rt, M - 1);
      if (a_rows) m = max(a_rows[m], 0);
      aoff[j] = (uint32_t)(((a_ld > 0 ? (size_t)m * KC : (size_t)m * K) + 8 * ((lane & 7) ^ swz(rt))) * 2);
    }
    int a_rd[4];                                          // this lane's fragment of step s inside a row tile
#pragma unroll
    for (int st = 0; st < 4; ++st) a_rd[st] = lr * 128 + (((4 * lg + st) ^ swz(lr)) << 4);
    const size_t a_cs = (a_ld > 0 ? (size_t)a_ld * KC : (size_t)KC) * 2;          // bytes between chunks
    const unsigned char* a_base = reinterpret_cast<const unsigned char*>(A);
    const int n0u = ni * (128 * NB) + lw * (32 * NB);     // n0 of the wave served, known to be wave-uniform
    const unsigned char* w_base[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int blk = min((n0u + nb * 32) >> 5, (N >> 5) - 1);   // clamped: computed, never stored
      w_base[nb] = reinterpret_cast<const unsigned char*>(W) + (size_t)blk * 4096;
    }
    const size_t W_CHUNK = (size_t)(N >> 5) * 4096;       // bytes between chunks of the packed weights
    const uint32_t lane16 = (uint32_t)lane * 16;
    // load l of a chunk: l < MT activation quarter-tiles, then the weights (column block, step)
    auto issue_one = [&](int l, int c, uint32_t sb) {
      if (l < MT) {
        load_to_lds16_sbase<0>(a_base + (size_t)c * a_cs, aoff[l], sb + (lw + 4 * l) * 1024);
      } else {
        const int nb = (l - MT) >> 2, st = (l - MT) & 3;
        const unsigned char* src = w_base[nb] + (size_t)c * W_CHUNK;
        const uint32_t dst = sb + A_STAGE + (lw * NB + nb) * 4096;
        // the constant is added to the global and to the LDS address alike
        if (st == 0) load_to_lds16_sbase<0>(src, lane16, dst);
        else if (st == 1) load_to_lds16_sbase<1024>(src, lane16, dst);
        else if (st == 2) load_to_lds16_sbase<2048>(src, lane16, dst);
        else load_to_lds16_sbase<3072>(src, lane16, dst);
      }
    };
    // The loads are issued by four waves of their own.  (Issued by the computing waves between their
    // MFMAs, every load costs the wave a dozen scalar instructions for base, LDS address and M0, and
    // a wave issues in order: the matrix core idles meanwhile.  A second wave per SIMD issues them
    // in the shadow of the first one's MFMAs.)  Loading wave 4 + w brings in the activation
    // quarter-tiles w, w + 4, ... and the weights of computing wave w; chunk c + 2 goes out once
    // every wave has passed the barrier of chunk c, i.e. is done with chunk c - 1, whose stage it takes.
    const int nc = c_end - c_begin;
    if (loader) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
        if (u < nc)
#pragma unroll
          for (int l = 0; l < LOADS; ++l) issue_one(l, c_begin + u, lds0 + u * STAGE);
      int stage = 2;
      for (int c = 0; c < nc; ++c) {
        // chunk c has landed (this wave's part; the barrier covers the other waves'), chunk c + 1
        // stays in flight
        if (c + 1 < nc) wait_loads_but<LOADS>();
        else wait_loads_but<0>();
        __syncthreads();
        if (c + 2 < nc) {
#pragma unroll
          for (int l = 0; l < LOADS; ++l) issue_one(l, c_begin + c + 2, lds0 + stage * STAGE);
        }
        stage = stage + 1 == RING ? 0 : stage + 1;
      }
      __syncthreads();
      return;
    }
    // The computing waves run the chunks as one stream of 16-wide steps.  Fragment reads go one MFMA
    // group ahead of their use, also across the chunk boundary: when the last step of a chunk starts,
    // all of that chunk's fragments are in registers, so the barrier that says "chunk c + 1 has landed"
    // sits there, and the last step's MFMAs cover the first reads of chunk c + 1.  (For the loading
    // waves the same barrier says that nobody reads chunk c's stage any more.)
    bf16x8_t af[2][MT], wf[2][NB];
    auto read_frag = [&](int stage, int st, int i) {
      const unsigned char* sa = lds + stage * STAGE;
      af[st & 1][i] = *reinterpret_cast<const bf16x8_t*>(sa + i * 4096 + a_rd[st]);
      if (i < NB)
        wf[st & 1][i] = *reinterpret_cast<const bf16x8_t*>(sa + A_STAGE + (wave_u * NB + i) * 4096 + lane * 16 + st * 1024);
    };
    static_assert(NB <= MT, "weight fragments ride along with the first NB activation fragments");
    if (nc > 0) {                                         // (uniform: the loading waves count the same barriers)
      __syncthreads();                                    // chunk 0 has landed
#pragma unroll
      for (int i = 0; i < MT; ++i) read_frag(0, 0, i);
    }
    int stage = 0;
    for (int c = 0; c < nc; ++c) {
      const int stage_next = stage + 1 == RING ? 0 : stage + 1;
      const bool more = c + 1 < nc;
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        if (st == 3 && more) __syncthreads();             // chunk c + 1 has landed; chunk c is in registers
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          if (st < 3) read_frag(stage, st + 1, i);
          else if (more) read_frag(stage_next, 0, i);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            acc[i][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st & 1][i], wf[st & 1][nb], acc[i][nb], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      stage = stage_next;
    }
    __syncthreads();                                      // the epilogues reuse the LDS
  } else {
  // weight pointers (clamped: out-of-range column blocks are computed but never stored)
  const u32x4_t* wp[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    if (TILED) {
      int blk = min((n0 + nb * 32) >> 5, (N >> 5) - 1);
      wp[nb] = reinterpret_cast<const u32x4_t*>(W) + (size_t)blk * 256 + lane;
    } else {
      int n = min(n0 + nb * 32 + lr, N - 1);
      wp[nb] = reinterpret_cast<const u32x4_t*>(W + (size_t)n * K + 32 * lg);
    }
  }
  const size_t W_CHUNK = TILED ? (size_t)(N >> 5) * 256 : KC * 2 / 16;   // u32x4_t between chunks of a lane's stream
  constexpr int W_STEP = TILED ? 64 : 1;               // u32x4_t between the steps of a chunk

  // activation staging: thread handles MT pieces of 16 B; piece p -> row p/8, 16-byte column p%8
  const bf16_t* ap[MT];
  int a_lds[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int p = tid + 256 * WM * i;
    int r = p >> 3, c16 = p & 7;
    int m = min(mt0 + r, M - 1);
    if (a_rows) m = max(a_rows[m], 0);
    ap[i] = A + (a_ld > 0 ? (size_t)m * KC : (size_t)m * K) + c16 * 8;
    a_lds[i] = r * A_ROW_BYTES + c16 * 16;
  }
  // activations: row-major [M][K] (a_ld == 0), or chunk-major [K/64][a_ld][64] where the rows of
  // one 64-wide k chunk are contiguous (row-major puts them 2K bytes apart, which lands every row
  // of a chunk on the same L2 channel when all workgroups walk the chunks in step)
  const size_t a_cs = a_ld > 0 ? (size_t)a_ld * KC : (size_t)KC;
  constexpr int A_BUF = WM * MT * 32 * A_ROW_BYTES;

  u32x4_t wreg[D][NB][4];
  u32x4_t areg[D][MT];

  // Every iteration issues the same loads (chunk indices past the split are clamped to its last
  // chunk, an L2 hit, and their activations are zeroed so they add nothing): with a fixed number
  // of loads in flight the compiler can wait for exactly the chunk it needs.
  const int c_last = max(c_end - 1, c_begin);
  const u32x4_t zero4 = {0u, 0u, 0u, 0u};
  // prologue: chunks c_begin .. c_begin+D-1
#pragma unroll
  for (int u = 0; u < D; ++u) {
    const int c = c_begin + u;
    const int cc = min(c, c_last);
#pragma unroll
    for (int i = 0; i < MT; ++i) areg[u][i] = *reinterpret_cast<const u32x4_t*>(ap[i] + (size_t)cc * a_cs);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int s = 0; s < 4; ++s) wreg[u][nb][s] = wp[nb][(size_t)cc * W_CHUNK + s * W_STEP];
  }
#pragma unroll
  for (int i = 0; i < MT; ++i)
    *reinterpret_cast<u32x4_t*>(lds + a_lds[i]) = c_begin < c_end ? areg[0][i] : zero4;
  __syncthreads();

  const int n_iter = (c_end - c_begin + D - 1) / D;   // groups of D chunks, the last one zero-padded
  for (int it = 0; it < n_iter; ++it) {
#pragma unroll
    for (int u = 0; u < D; ++u) {
      const int c = c_begin + it * D + u;
      const int buf = u & 1;                            // D is even
      const unsigned char* abase = lds + buf * A_BUF + (wm * MT * 32 + lr) * A_ROW_BYTES + 64 * lg;
      // Fragment reads run one MFMA step ahead and are pinned between the MFMA groups (scheduling
      // barriers), so each read has MT*NB MFMAs of cover before its first use.
      bf16x8_t af[2][MT];
#pragma unroll
      for (int i = 0; i < MT; ++i) af[0][i] = *reinterpret_cast<const bf16x8_t*>(abase + i * 32 * A_ROW_BYTES);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          if (s < 3)
            af[(s + 1) & 1][i] = *reinterpret_cast<const bf16x8_t*>(abase + i * 32 * A_ROW_BYTES + 16 * (s + 1));
          {
            // refill of ring slot u with chunk c+D, one load per MFMA group (a burst after the
            // MFMAs would hold the wave at the memory pipeline's address queue while the matrix
            // cores idle): the activation registers are free (stored to LDS a chunk ago), the
            // weight registers of step s-1 were consumed by the previous step
            const int cc = min(c + D, c_last);
            if (s == 0) areg[u][i] = *reinterpret_cast<const u32x4_t*>(ap[i] + (size_t)cc * a_cs);
            else if (i < NB) wreg[u][i][s - 1] = wp[i][(size_t)cc * W_CHUNK + (s - 1) * W_STEP];
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            bf16x8_t bfr = __builtin_bit_cast(bf16x8_t, wreg[u][nb][s]);
            acc[i][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s & 1][i], bfr, acc[i][nb], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // activations of chunk c+1 (ring slot u+1) -> the other LDS buffer
#pragma unroll
      for (int i = 0; i < MT; ++i)
        *reinterpret_cast<u32x4_t*>(lds + (buf ^ 1) * A_BUF + a_lds[i]) =
            c + 1 < c_end ? areg[(u + 1) % D][i] : zero4;   // zeroed at use, not at load
      // the last step's weight registers of ring slot u
      {
        const int cc = min(c + D, c_last);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) wreg[u][nb][3] = wp[nb][(size_t)cc * W_CHUNK + 3 * W_STEP];
      }
      __syncthreads();
    }
  }
  }   // register-ring path

  // epilogue: lane holds column n, rows 8*(v/4) + 4*lg + v%4 of each 32x32 tile
  if (EPI == 0 || EPI == 3) {
    float* o = out + (size_t)z * M * N;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n = n0 + nb * 32 + lr;
      if (n0 + nb * 32 < N) {
#pragma unroll
        for (int i = 0; i < MT; ++i) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            int m = m0 + i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
            if (m < M) o[(size_t)m * N + n] = acc[i][nb][v];
          }
        }
      }
    }
  }
  if ((EPI == 1 || EPI == 3) && RING > 0) {
    // arg-max epilogue of the large tile (LM head at many tree rows; needs splits == 1): per row the
    // maximum over this workgroup's columns, lowest column on ties; `out` receives [n_tiles][M] pairs
    // (value, column as int bits) and the logits themselves are never written.  A lane holds one
    // column of 16 rows per MFMA tile, so the maximum along a row is a reduction across lanes: each
    // wave transposes its tile through its own slice of the (now idle) ring and every lane then
    // scans whole rows with 16-byte reads.  (Butterfly shuffles cost ten LDS round trips per row.)
    constexpr int ROWS = MT * 32, LD = 36;                  // 36 words: 16-byte aligned rows, 2-way conflicts at most
    float* tr = reinterpret_cast<float*>(lds) + wave * (ROWS * LD);
    float best[(ROWS + 63) / 64];
    int bi[(ROWS + 63) / 64];
#pragma unroll
    for (int q = 0; q < (ROWS + 63) / 64; ++q) { best[q] = -INFINITY; bi[q] = 0x7fffffff; }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int nbase = n0 + nb * 32;
      if (draw_pos) {   // sample matching: the row draws its next token, arg-max of logit + Gumbel noise
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int rl = i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
            tr[rl * LD + lr] = acc[i][nb][v] +
                               gumbel_noise(seed, (uint32_t)draw_pos[min(m0 + rl, M - 1)], (uint32_t)(nbase + lr));
          }
      } else {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) tr[(i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3)) * LD + lr] = acc[i][nb][v];
      }
      if (nbase < N) {
#pragma unroll
        for (int q = 0; q < (ROWS + 63) / 64; ++q) {
          const int rl = q * 64 + lane;
          if (rl < ROWS) {
            f32x4_t x[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) x[c] = *reinterpret_cast<const f32x4_t*>(tr + rl * LD + 4 * c);
#pragma unroll
            for (int c = 0; c < 32; ++c)   // columns ascend: ties keep the lower one
              if (x[c >> 2][c & 3] > best[q]) { best[q] = x[c >> 2][c & 3]; bi[q] = nbase + c; }
          }
        }
      }
    }
    __syncthreads();                                        // every wave is done with its slice
    float* red = reinterpret_cast<float*>(lds);             // [4 waves][ROWS][2]
#pragma unroll
    for (int q = 0; q < (ROWS + 63) / 64; ++q) {
      const int rl = q * 64 + lane;
      if (rl < ROWS) {
        red[(wn * ROWS + rl) * 2 + 0] = best[q];
        red[(wn * ROWS + rl) * 2 + 1] = __int_as_float(bi[q]);
      }
    }
    __syncthreads();
    for (int rl = tid; rl < ROWS; rl += 256) {
      float bv = red[rl * 2];
      int bj = __float_as_int(red[rl * 2 + 1]);
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float ov = red[(w * ROWS + rl) * 2];
        const int oi = __float_as_int(red[(w * ROWS + rl) * 2 + 1]);
        if (ov > bv || (ov == bv && oi < bj)) { bv = ov; bj = oi; }
      }
      const int m = mt0 + rl;
      float* pairs = EPI == 3 ? out2 : out;
      if (m < M) {
        pairs[((size_t)ni * M + m) * 2 + 0] = bv;
        pairs[((size_t)ni * M + m) * 2 + 1] = __int_as_float(bj);
      }
    }
  } else if (EPI == 1 || EPI == 3) {
    // arg-max epilogue of the small tiles: the same result by butterfly shuffles (their LDS holds no
    // transposed tile)
    float* red = reinterpret_cast<float*>(lds);            // [4 waves][MT*32 rows][2]
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float best = -INFINITY;
        int bi = 0x7fffffff;
        // sample matching: the row draws its next token, arg-max of logit + Gumbel noise
        const uint32_t pos =
            draw_pos ? (uint32_t)draw_pos[min(m0 + i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3), M - 1)] : 0u;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const int n = n0 + nb * 32 + lr;
          float x = acc[i][nb][v];
          if (draw_pos) x += gumbel_noise(seed, pos, (uint32_t)n);
          if (n0 + nb * 32 < N && (x > best || (x == best && n < bi))) { best = x; bi = n; }
        }
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) {                  // over the 32 columns of a lane half
          float ov = __shfl_xor(best, o, 64);
          int oi = __shfl_xor(bi, o, 64);
          if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
        }
        if (lr == 0) {
          const int rl = i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
          red[(wn * MT * 32 + rl) * 2 + 0] = best;
          red[(wn * MT * 32 + rl) * 2 + 1] = __int_as_float(bi);
        }
      }
    }
    __syncthreads();
    for (int rl = tid; rl < MT * 32; rl += 256) {
      float best = red[rl * 2];
      int bi = __float_as_int(red[rl * 2 + 1]);
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        float ov = red[(w * MT * 32 + rl) * 2];
        int oi = __float_as_int(red[(w * MT * 32 + rl) * 2 + 1]);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
      }
      const int m = mt0 + rl;
      float* pairs = EPI == 3 ? out2 : out;
      if (m < M) {
        pairs[((size_t)ni * M + m) * 2 + 0] = best;
        pairs[((size_t)ni * M + m) * 2 + 1] = __int_as_float(bi);
      }
    }
  }
  if (EPI == 2) {
    // SwiGLU epilogue (fused gate/up projection; needs splits == 1): the weight rows alternate
    // in blocks of 32 between gate and up, so output column block 2j is gate block j and 2j+1 is
    // up block j.  `out` is the bf16 activation matrix [M][N/2]: act = silu(gate) * up.
    bf16_t* act = reinterpret_cast<bf16_t*>(out);
    const int ff = N >> 1;
    if (NB == 2) {   // both blocks in this lane's registers
      if (n0 < N) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int m = m0 + i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
            const float g = acc[i][0][v], u = acc[i][NB - 1][v];
            if (m < M) act[(size_t)m * ff + (n0 >> 1) + lr] = (bf16_t)silu_mul(g, u);
          }
      }
    } else {         // the odd wave of a pair holds the up block: hand it over through LDS
      float* ex = reinterpret_cast<float*>(lds);              // [2 pairs][MT*32 rows][32]
      if (wn & 1) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            ex[((wn >> 1) * MT * 32 + i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3)) * 32 + lr] = acc[i][0][v];
      }
      __syncthreads();
      if (!(wn & 1) && n0 < N) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int rl = i * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
            const int m = m0 + rl;
            const float g = acc[i][0][v], u = ex[((wn >> 1) * MT * 32 + rl) * 32 + lr];
            if (m < M) act[(size_t)m * ff + (n0 >> 1) + lr] = (bf16_t)silu_mul(g, u);
          }
      }
    }
  }
}

// Two entry points over the same body.  The small-tile one (<= 4 row tiles, one column block per
// wave) leaves occupancy to the compiler.  The large-tile one tells it that one wave per SIMD is
// all it will ever get, so registers go to prefetching.  (A 512-thread variant with two row groups
// per workgroup and two waves per SIMD was measured and was not faster.)
template <int MT, int NB, int D, bool TILED, int EPI>
__global__ __launch_bounds__(256) void k_gemm_bf16(const bf16_t* __restrict__ A, const int32_t* __restrict__ a_rows,
                                                   const bf16_t* __restrict__ W, float* __restrict__ out, int M,
                                                   int N, int K, int splits, int m_tiles, int n_tiles, int a_ld,
                                                   float* __restrict__ out2, const int32_t* __restrict__ draw_pos,
                                                   uint32_t seed) {
  extern __shared__ __align__(16) unsigned char lds[];   // 2 buffers of MT*32 rows * A_ROW_BYTES
  gemm_bf16_body<MT, NB, D, TILED, 1, EPI>(lds, A, a_rows, W, out, M, N, K, splits, m_tiles, n_tiles, a_ld, out2,
                                           draw_pos, seed);
}

template <int MT, int NB, int D, bool TILED, int EPI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_gemm_bf16_big(
    const bf16_t* __restrict__ A, const int32_t* __restrict__ a_rows, const bf16_t* __restrict__ W,
    float* __restrict__ out, int M, int N, int K, int splits, int m_tiles, int n_tiles, int a_ld,
    float* __restrict__ out2) {
  extern __shared__ __align__(16) unsigned char lds[];
  gemm_bf16_body<MT, NB, D, TILED, 1, EPI>(lds, A, a_rows, W, out, M, N, K, splits, m_tiles, n_tiles, a_ld, out2,
                                           nullptr, 0u);
}

// Large tile with the LDS ring: one workgroup of eight waves per CU owns (almost) the whole LDS;
// waves 0..3 compute, waves 4..7 load (two waves per SIMD, 256 registers each: the 160 accumulator
// registers of a 5 x 2 tile fit).
constexpr int RING_STAGES = 3;
template <int MT, int NB>
constexpr size_t ring_lds_bytes() { return (size_t)RING_STAGES * (MT * 4096 + 4 * NB * 4096); }

template <int MT, int NB, int EPI>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_gemm_bf16_ring(
    const bf16_t* __restrict__ A, const int32_t* __restrict__ a_rows, const bf16_t* __restrict__ W,
    float* __restrict__ out, int M, int N, int K, int splits, int m_tiles, int n_tiles, int a_ld,
    float* __restrict__ out2, const int32_t* __restrict__ draw_pos, uint32_t seed) {
  extern __shared__ __align__(16) unsigned char lds[];
  gemm_bf16_body<MT, NB, 2, true, 1, EPI, RING_STAGES>(lds, A, a_rows, W, out, M, N, K, splits, m_tiles, n_tiles, a_ld,
                                                      out2, draw_pos, seed);
}

// ---- fp32: 64x64 tile, 16-deep k steps, 256 threads, 4x4 outputs per thread -----------------------
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A, const int32_t* __restrict__ a_rows,
                                                  const float* __restrict__ W, float* __restrict__ out, int M,
                                                  int N, int K) {
  __shared__ float As[16][65];
  __shared__ float Ws[16][65];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      int r = i >> 4, kk = i & 15;
      int m = m0 + r, n = n0 + r, k = k0 + kk;
      float av = 0.f, wv = 0.f;
      if (m < M && k < K) {
        int pm = a_rows ? max(a_rows[m], 0) : m;
        av = A[(size_t)pm * K + k];
      }
      if (n < N && k < K) wv = W[(size_t)n * K + k];
      As[kk][r] = av;
      Ws[kk][r] = wv;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) out[(size_t)m * N + n] = acc[i][j];
    }
}

// row-major [N][K] -> tiles of 32 rows x 64 k stored as [chunk][row block][step][lane][8]
__global__ void k_pack_weight(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N, int K) {
  const size_t piece = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte piece
  const size_t total = (size_t)N * K / 8;
  if (piece >= total) return;
  const int chunks = K / KC;
  const int lane = piece & 63, s = (piece >> 6) & 3;
  const size_t tile = piece >> 8;
  const int nblk = N >> 5;
  const int blk = (int)(tile % nblk);
  const int c = (int)(tile / nblk);
  const int n = blk * 32 + (lane & 31);
  const int k = c * KC + 32 * (lane >> 5) + 8 * s;
  reinterpret_cast<uint4*>(dst)[piece] = *reinterpret_cast<const uint4*>(src + (size_t)n * K + k);
}

// The ring kernels use more dynamic LDS than a kernel gets by default: raise the limit once per
// kernel (gemm_prepare does it for all of them when a context is created, so that no launch inside
// a stream capture is the first one).
template <int MT, int NB, int EPI>
hipError_t ring_allow_lds() {
  static const hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_bf16_ring<MT, NB, EPI>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)ring_lds_bytes<MT, NB>());
  return attr;
}

// launch, with a profiling scope's events attached to the kernel when there are any
template <typename Kern, typename... Args>
void launch_kernel(Kern kern, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
  if (g_launch_events.start) {
    hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)lds, st, g_launch_events.start, g_launch_events.stop, 0, args...);
    g_launch_events = LaunchEvents{};
  } else {
    hipLaunchKernelGGL(kern, grid, block, lds, st, args...);
  }
}

template <int MT, int NB, bool TILED = true, int D = (MT * NB >= 8 ? 2 : 4), int EPI = 0>
hipError_t launch_bf16(hipStream_t st, const void* A, const int32_t* a_rows, const void* W, float* out, int M,
                       int N, int K, const GemmPlan& p, int a_ld = 0, float* out2 = nullptr,
                       const int32_t* draw_pos = nullptr, uint32_t seed = 0) {
  int total = p.m_tiles * p.n_tiles * p.splits;
  int per_xcd = (total + 7) / 8;
  size_t lds = 2 * (size_t)MT * 32 * A_ROW_BYTES;
  if constexpr (MT * NB >= 8 && TILED) {
    auto kern = k_gemm_bf16_ring<MT, NB, EPI>;
    const hipError_t attr = ring_allow_lds<MT, NB, EPI>();
    if (attr != hipSuccess) return attr;
    const size_t ring_bytes = ring_lds_bytes<MT, NB>();
    launch_kernel(kern, dim3(per_xcd * 8), dim3(512), ring_bytes, st, (const bf16_t*)A, a_rows, (const bf16_t*)W, out,
                  M, N, K, p.splits, p.m_tiles, p.n_tiles, a_ld, out2, draw_pos, seed);
  } else if constexpr (MT * NB >= 8)
    launch_kernel(k_gemm_bf16_big<MT, NB, D, TILED, EPI>, dim3(per_xcd * 8), dim3(256), lds, st, (const bf16_t*)A,
                  a_rows, (const bf16_t*)W, out, M, N, K, p.splits, p.m_tiles, p.n_tiles, a_ld, out2);
  else
    launch_kernel(k_gemm_bf16<MT, NB, D, TILED, EPI>, dim3(per_xcd * 8), dim3(256), lds, st, (const bf16_t*)A, a_rows,
                  (const bf16_t*)W, out, M, N, K, p.splits, p.m_tiles, p.n_tiles, a_ld, out2, draw_pos, seed);
  return hipGetLastError();
}

}  // namespace

thread_local LaunchEvents g_launch_events;

hipError_t gemm_prepare() {
  hipError_t e = ring_allow_lds<4, 2, 0>();
  if (e == hipSuccess) e = ring_allow_lds<4, 2, 2>();
  if (e == hipSuccess) e = ring_allow_lds<5, 2, 0>();
  if (e == hipSuccess) e = ring_allow_lds<5, 2, 2>();
  if (e == hipSuccess) e = ring_allow_lds<4, 2, 1>();
  if (e == hipSuccess) e = ring_allow_lds<5, 2, 1>();
  return e;
}

GemmPlan gemm_plan(int dtype, int M, int N, int K) {
  GemmPlan p;
  p.wm = 1;
  if (dtype == ESP_F32) {
    p.splits = 1; p.mt = 2; p.nb = 2; p.m_tiles = (M + 63) / 64; p.n_tiles = (N + 63) / 64;
    return p;
  }
  const int tiles32 = (M + 31) / 32;
  const int max_s = std::max(1, K / (KC * 8));    // at least 8 chunks per split
  if (tiles32 <= 4) {
    // up to 128 rows: one row tile per workgroup, 128 columns.
    // split-K from (N, K) only: as many parts as keep the launch within 256 workgroups, one per CU
    // (288 workgroups on the QKV shape leave 32 CUs with two: 24 us against 21 us at 68 rows)
    p.mt = tiles32; p.nb = 1; p.m_tiles = 1;
    p.n_tiles = (N + 127) / 128;
    p.splits = std::max(1, std::min(std::min(256 / p.n_tiles, max_s), 8));
  } else {
    // more rows: up to 5 row tiles and 256 columns per workgroup, one workgroup per CU (the
    // accumulators fill the register file); split-K fills the 256 CUs without spilling into a
    // second, mostly empty round (measured: 240 workgroups beat 288 by 1.6x on the QKV shape)
    p.nb = 2;
    p.m_tiles = (tiles32 + 4) / 5;
    p.mt = (tiles32 + p.m_tiles - 1) / p.m_tiles;
    p.n_tiles = (N + 255) / 256;
    p.splits = std::max(1, std::min(std::min(256 / (p.m_tiles * p.n_tiles), max_s), 8));
  }
  return p;
}

namespace {

// arg-max over the per-tile partials written by the AMAX epilogue: one workgroup per row
__global__ __launch_bounds__(256) void k_argmax_tiles(const float* __restrict__ part, int n_tiles, int M,
                                                      const int32_t* __restrict__ row_map, int32_t* __restrict__ out,
                                                      const int32_t* __restrict__ out_index) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int dst = out_index ? out_index[blockIdx.x] : (int)blockIdx.x;
  if (dst < 0) return;
  const int m = row_map ? max(row_map[blockIdx.x], 0) : (int)blockIdx.x;   // row of the pair table
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int t = threadIdx.x; t < n_tiles; t += 256) {
    float v = part[((size_t)t * M + m) * 2];
    int i = __float_as_int(part[((size_t)t * M + m) * 2 + 1]);
    if (v > best || (v == best && i < bi)) { best = v; bi = i; }
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

}  // namespace

// LM head with the arg-max taken in the GEMM epilogue (bf16, packed weights): scratch holds
// n_tiles * M (value, column) pairs; out[out_index[m]] = arg-max of row m.  Up to 128 rows the
// logits of all rows can be written as well (logits_out); above, the large-tile kernel takes the
// arg-max only and the [rows, vocab] logits are never written.
bool gemm_argmax_supported(int dtype, int M, int N, int K, bool with_logits) {
  if (dtype != ESP_BF16) return false;
  GemmPlan p = gemm_plan(dtype, M, N, K);
  if (p.splits != 1) return false;
  if (p.nb == 1 && p.m_tiles == 1) return true;
  return !with_logits && p.nb == 2 && p.mt >= 3 && p.mt <= 5;
}
size_t gemm_argmax_scratch_floats(int M, int N) { return (size_t)((N + 127) / 128) * M * 2; }

hipError_t launch_gemm_argmax(hipStream_t st, const void* A, const int32_t* a_rows, const void* W, int M, int N,
                              int K, float* scratch, int32_t* out, const int32_t* out_index, int a_ld,
                              float* logits_out, const int32_t* arg_rows, int n_arg, const int32_t* draw_pos,
                              uint32_t seed) {
  GemmPlan p = gemm_plan(ESP_BF16, M, N, K);
  hipError_t e = hipErrorInvalidValue;
  // without logits_out: pairs only (the logits are never written); with it: the fp32 logits of all M
  // rows as well
#define ESP_AMAX_CASE(MT_)                                                                                     \
  case MT_:                                                                                                    \
    e = logits_out ? launch_bf16<MT_, 1, true, 4, 3>(st, A, a_rows, W, logits_out, M, N, K, p, a_ld, scratch,  \
                                                     draw_pos, seed)                                           \
                   : launch_bf16<MT_, 1, true, 4, 1>(st, A, a_rows, W, scratch, M, N, K, p, a_ld, nullptr,     \
                                                     draw_pos, seed);                                          \
    break;
  if (p.nb == 2) {   // many rows: large tiles, pairs only
    if (logits_out) return hipErrorInvalidValue;
    if (p.mt == 3) e = launch_bf16<3, 2, true, 4, 1>(st, A, a_rows, W, scratch, M, N, K, p, a_ld, nullptr, draw_pos, seed);
    else if (p.mt == 4) e = launch_bf16<4, 2, true, 2, 1>(st, A, a_rows, W, scratch, M, N, K, p, a_ld, nullptr, draw_pos, seed);
    else if (p.mt == 5) e = launch_bf16<5, 2, true, 2, 1>(st, A, a_rows, W, scratch, M, N, K, p, a_ld, nullptr, draw_pos, seed);
  } else {
    switch (p.mt) {
      ESP_AMAX_CASE(1)
      ESP_AMAX_CASE(2)
      ESP_AMAX_CASE(3)
      ESP_AMAX_CASE(4)
    }
  }
#undef ESP_AMAX_CASE
  if (e != hipSuccess) return e;
  // out[out_index[i]] = arg-max of row arg_rows[i] (or of row i), i < n_arg
  hipLaunchKernelGGL(k_argmax_tiles, dim3(n_arg), dim3(256), 0, st, scratch, p.n_tiles, M, arg_rows, out, out_index);
  return hipGetLastError();
}

// Fused gate/up projection + SwiGLU (bf16, packed weights whose rows alternate in blocks of 32
// between gate and up): act[M][ff] = silu(A Wg^T) * (A Wu^T), one pass over K per workgroup.
hipError_t launch_gemm_swiglu(hipStream_t st, const void* A, const void* W, void* act, int M, int ff, int K) {
  if (M <= 0) return hipSuccess;
  GemmPlan p = gemm_plan(ESP_BF16, M, 2 * ff, K);
  p.splits = 1;
  float* out = reinterpret_cast<float*>(act);
#define ESP_GU_CASE(MT_, NB_)                                                                           \
  if (p.mt == MT_ && p.nb == NB_)                                                                       \
    return launch_bf16<MT_, NB_, true, (MT_ * NB_ >= 8 ? 2 : 4), 2>(st, A, nullptr, W, out, M, 2 * ff, K, p);
  ESP_GU_CASE(1, 1)
  ESP_GU_CASE(2, 1)
  ESP_GU_CASE(3, 1)
  ESP_GU_CASE(4, 1)
  ESP_GU_CASE(3, 2)
  ESP_GU_CASE(4, 2)
  ESP_GU_CASE(5, 2)
#undef ESP_GU_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_pack_weight(hipStream_t st, const void* src, void* dst, int N, int K) {
  size_t pieces = (size_t)N * K / 8;
  hipLaunchKernelGGL(k_pack_weight, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, (const bf16_t*)src,
                     (bf16_t*)dst, N, K);
  return hipGetLastError();
}

hipError_t launch_gemm(hipStream_t st, int dtype, const void* A, const int32_t* a_rows, const void* W,
                       float* out, int M, int N, int K, const GemmPlan& p, bool w_packed, int a_ld) {
  if (M <= 0) return hipSuccess;
  if (dtype == ESP_F32) {
    hipLaunchKernelGGL(k_gemm_f32, dim3(p.n_tiles, p.m_tiles), dim3(256), 0, st, (const float*)A, a_rows,
                       (const float*)W, out, M, N, K);
    return hipGetLastError();
  }
#define ESP_GEMM_CASE(MT_, NB_)                                                                  \
  if (p.mt == MT_ && p.nb == NB_)                                                                \
    return w_packed ? launch_bf16<MT_, NB_, true>(st, A, a_rows, W, out, M, N, K, p, a_ld)       \
                    : launch_bf16<MT_, NB_, false>(st, A, a_rows, W, out, M, N, K, p, a_ld);
  ESP_GEMM_CASE(1, 1)
  ESP_GEMM_CASE(2, 1)
  ESP_GEMM_CASE(3, 1)
  ESP_GEMM_CASE(4, 1)
  ESP_GEMM_CASE(1, 2)
  ESP_GEMM_CASE(2, 2)
  ESP_GEMM_CASE(3, 2)
  ESP_GEMM_CASE(4, 2)
  ESP_GEMM_CASE(5, 2)
#undef ESP_GEMM_CASE
  return hipErrorInvalidValue;
}
