// Tree logic kept on the device: block descriptor from parent pointers, greedy acceptance + KV
// commit, row lists for the proposal pass, pruning + dynamic tree construction
// (paper Sec. 2 Eq. 3, Sec. 3.3-3.5, Alg. 1, App. C, App. E).  One workgroup per sequence;
// everything is integer work except the fp32 products of Alg. 1.
#include "esp_internal.h"

namespace {

constexpr int MAX_ANC_WORDS = ESP_MAX_ROWS_PER_SEQ / 64;
constexpr int MAXC = 4096;   // candidates Alg. 1 may create (root included)

__device__ __forceinline__ bool kv_seq_ok(const KvDev& kv, int seq, int n_rows, int rows_per_seq) {
  int L = kv.len[seq];
  int base = kv.base[seq];
  int cap = kv.seq_cap[seq];
  return L >= 0 && L <= kv.len_bound && n_rows >= 0 && n_rows <= rows_per_seq && L + n_rows <= cap &&
         base >= 0 && (base & 63) == 0 && (int64_t)base + cap <= kv.capacity;
}

// Derives every per-row array of one sequence from tok/parent/n_nodes of its node rows.
// Called by all threads of the workgroup; tok/parent of the node rows must be visible.
__device__ void finalize_block(int seq, int rows_per_seq, int k, int layout, int anc_words, int32_t* n_rows,
                               int n_nodes, int32_t* tok, int32_t* parent, int32_t* depth, int32_t* mask_j,
                               int32_t* attach, uint64_t* anc, int32_t* status, int* s_bad) {
  const size_t r0 = (size_t)seq * rows_per_seq;
  const int owners = k == 0 ? 0 : (layout == ESP_LAYOUT_PER_NODE ? n_nodes : 1);
  const int total = n_nodes + owners * k;
  if (threadIdx.x == 0) *s_bad = (n_nodes < 1 || total > rows_per_seq || (total + 63) / 64 > anc_words) ? 1 : 0;
  __syncthreads();
  if (!*s_bad) {
    for (int i = threadIdx.x; i < n_nodes; i += blockDim.x) {
      uint64_t bits[MAX_ANC_WORDS];
      for (int w = 0; w < anc_words; ++w) bits[w] = 0;
      int c = i, dep = 0;
      bool bad = false;
      for (int step = 0; step <= n_nodes; ++step) {
        bits[c >> 6] |= 1ull << (c & 63);
        int p = parent[r0 + c];
        if (c == 0) { bad = p != -1; break; }
        if (p < 0 || p >= c) { bad = true; break; }
        c = p;
        ++dep;
      }
      if (bad) atomicExch(s_bad, 1);
      depth[r0 + i] = dep;
      mask_j[r0 + i] = 0;
      attach[r0 + i] = i;
      for (int w = 0; w < anc_words; ++w) anc[(r0 + i) * anc_words + w] = bits[w];
    }
  }
  __syncthreads();
  if (*s_bad) {
    if (threadIdx.x == 0) { atomicOr(status, ESP_DEV_BAD_TREE); n_rows[seq] = 0; }
    return;
  }
  // mask rows: chain j = 1..k of owner a sits at n_nodes + a*k + (j-1)
  for (int t = threadIdx.x; t < owners * k; t += blockDim.x) {
    int a = t / k, j = t % k + 1;
    int row = n_nodes + t;
    int first = row - (j - 1);
    for (int w = 0; w < anc_words; ++w) {
      uint64_t bits = anc[(r0 + a) * anc_words + w];
      // rows first..row of the chain
      int lo = max(first, w * 64), hi = min(row, w * 64 + 63);
      for (int c = lo; c <= hi; ++c) bits |= 1ull << (c & 63);
      anc[(r0 + row) * anc_words + w] = bits;
    }
    tok[r0 + row] = -1;
    parent[r0 + row] = j == 1 ? a : row - 1;
    depth[r0 + row] = depth[r0 + a] + j;
    mask_j[r0 + row] = j;
    attach[r0 + row] = a;
  }
  if (threadIdx.x == 0) n_rows[seq] = total;
}

__global__ __launch_bounds__(256) void k_block_from_tree(int rows_per_seq, int k, int layout, int anc_words,
                                                         int32_t* n_rows, const int32_t* n_nodes, int32_t* tok,
                                                         int32_t* parent, int32_t* depth, int32_t* mask_j,
                                                         int32_t* attach, uint64_t* anc, int32_t* status) {
  __shared__ int s_bad;
  const int seq = blockIdx.x;
  finalize_block(seq, rows_per_seq, k, layout, anc_words, n_rows, n_nodes[seq], tok, parent, depth, mask_j,
                 attach, anc, status, &s_bad);
}

// ---- greedy verification (Sec. 2 Eq. 3) -----------------------------------------------------------------
__global__ __launch_bounds__(256) void k_verify(BlockDev b, KvDev kv, const int32_t* __restrict__ g,
                                                int32_t* n_emit, int32_t* emit_tok, int32_t* accepted_row,
                                                int32_t* star_row) {
  __shared__ int s_next;
  const int seq = blockIdx.x;
  const size_t r0 = (size_t)seq * b.rows_per_seq;
  const int nn = b.n_nodes[seq], nr = b.n_rows[seq];
  int32_t* et = emit_tok + (size_t)seq * (ESP_MAX_MASKS + 1);
  int32_t* ar = accepted_row + (size_t)seq * (ESP_MAX_MASKS + 1);
  if (!kv_seq_ok(kv, seq, nr, b.rows_per_seq) || nn < 1 || nn > nr) {
    if (threadIdx.x == 0) { n_emit[seq] = 0; star_row[seq] = 0; }
    return;
  }
  int cur = 0, a = 0;
  if (threadIdx.x == 0) ar[0] = 0;
  while (a < ESP_MAX_MASKS) {
    if (threadIdx.x == 0) s_next = 0x7fffffff;
    __syncthreads();
    const int want = g[r0 + cur];
    for (int c = threadIdx.x; c < nn; c += blockDim.x)
      if (b.parent[r0 + c] == cur && b.tok[r0 + c] == want) atomicMin(&s_next, c);   // first match in row order
    __syncthreads();
    const int nxt = s_next;
    __syncthreads();
    if (nxt == 0x7fffffff) break;
    if (threadIdx.x == 0) { et[a] = b.tok[r0 + nxt]; ar[a + 1] = nxt; }
    cur = nxt;
    ++a;
  }
  if (threadIdx.x == 0) {
    et[a] = g[r0 + cur];
    n_emit[seq] = a + 1;
    star_row[seq] = cur;
    kv.len[seq] += a + 1;
  }
}

// moves the accepted rows' K/V to slots L+1.. in path order; one workgroup per (layer*kv_head, seq),
// one thread per feature, accepted rows processed in order (a destination can be a later source).
template <typename T>
__global__ void k_kv_commit(BlockDev b, KvDev kv, int n_kv, int hd, const int32_t* __restrict__ n_emit,
                            const int32_t* __restrict__ accepted_row) {
  const int seq = blockIdx.y;
  const int ne = n_emit[seq];
  if (ne < 2) return;
  const int layer = blockIdx.x / n_kv, kvh = blockIdx.x % n_kv;
  const int d = threadIdx.x;
  const int L = kv.len[seq] - ne;    // k_verify already advanced len
  const int64_t base = kv.base[seq];
  T* kp = (T*)kv.k + kv_plane(layer, kvh, n_kv, kv.capacity, hd);
  T* vp = (T*)kv.v + kv_plane(layer, kvh, n_kv, kv.capacity, hd);
  const int32_t* ar = accepted_row + (size_t)seq * (ESP_MAX_MASKS + 1);
  for (int i = 1; i < ne; ++i) {
    int64_t src = base + L + ar[i], dst = base + L + i;
    if (src == dst) continue;
    kp[k_off(dst, d, hd)] = kp[k_off(src, d, hd)];
    vp[v_off(dst, d, hd)] = vp[v_off(src, d, hd)];
  }
}

// rows whose logits seed the next tree (Sec. 3.3): mask rows aligned to the accepted position
__global__ void k_mask_rows(BlockDev b, const int32_t* star_row, const int32_t* n_emit, int32_t* a_rows,
                            int32_t* n_lists) {
  const int seq = blockIdx.x;
  const int k = b.k_masks;
  const int nn = b.n_nodes[seq], nr = b.n_rows[seq], ne = n_emit[seq];
  int lists = 0, first = 0;
  if (ne >= 1 && nn >= 1 && nr <= b.rows_per_seq) {
    if (b.layout == ESP_LAYOUT_PER_NODE) {
      int s = star_row[seq];
      if (s >= 0 && s < nn && nn * (k + 1) == nr) { lists = k; first = nn + s * k; }
    } else {
      int a = ne - 1;
      if (nn + k == nr && a < k) { lists = k - a; first = nn + a; }
    }
  }
  for (int i = threadIdx.x; i < k; i += blockDim.x)
    a_rows[seq * k + i] = i < lists ? seq * b.rows_per_seq + first + i : -1;
  if (threadIdx.x == 0) n_lists[seq] = lists;
}

// ---- pruning + dynamic tree (Alg. 1, Sec. 3.5) -----------------------------------------------------------
struct TreeLds {
  int32_t tok[MAXC];
  float prob[MAXC];
  int16_t par[MAXC];
  uint8_t dep[MAXC];
  uint8_t used[MAXC];        // has been in the node set N
  uint64_t key[MAXC];        // sort buffer
  int32_t frontier[ESP_MAX_TREE_NODES];
  int32_t expand[ESP_MAX_TREE_NODES];
  int32_t scan[256];
  int32_t n_total, n_frontier, n_expand, bad;
  int32_t n_surv, bin1, before1, bin2;   // select_best
  int32_t list_id[ESP_MAX_MASKS * ESP_MAX_TOPK];   // the sequence's Top-K' lists, staged once
  float list_p[ESP_MAX_MASKS * ESP_MAX_TOPK];
};

__device__ __forceinline__ uint64_t cand_key(float p, int creation) {
  // ascending key order = probability descending, then creation ascending
  return ((uint64_t)(~__float_as_uint(p)) << 32) | (uint32_t)creation;
}

__device__ void bitonic_sort(uint64_t* key, int n_pow2) {
  for (int size = 2; size <= n_pow2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = threadIdx.x; t < (n_pow2 >> 1); t += blockDim.x) {
        int lo = 2 * t - (t & (stride - 1));
        int hi = lo + stride;
        bool up = (lo & size) == 0;
        uint64_t a = key[lo], c = key[hi];
        if ((a > c) == up) { key[lo] = c; key[hi] = a; }
      }
      __syncthreads();
    }
  }
}

// exclusive scan of one value per thread over the 256-thread block; returns (prefix, total via *tot)
__device__ int block_excl_scan(int v, int32_t* buf, int* tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int x = __shfl_up(incl, o, 64);
    if (lane >= o) incl += x;
  }
  if (lane == 63) buf[wave] = incl;
  __syncthreads();
  const int w0 = buf[0], w1 = buf[1], w2 = buf[2], w3 = buf[3];
  *tot = w0 + w1 + w2 + w3;
  const int base = wave == 0 ? 0 : wave == 1 ? w0 : wave == 2 ? w0 + w1 : w0 + w1 + w2;
  __syncthreads();
  return base + incl - v;
}

// The T best (smallest key) of the eligible candidates 0..n-1, in key order, to out[0..m);
// returns m = min(T, eligible), or -1 when the shortcut below does not apply (the caller then
// sorts everything).  T <= 255.  Instead of sorting all candidates, a two-level histogram over the
// key's leading bits (the probability's exponent, then its top 8 mantissa bits) finds a prefix
// bound that at least T candidates meet; the few that meet it (T plus the occupants of one
// histogram cell, at most 256 or the shortcut is off) are ranked against each other directly.
// Keys are unique (they end in the creation index), so ranks are a permutation.
template <typename Elig>
__device__ int select_best(TreeLds& s, int n, int T, Elig eligible, int32_t* out) {
  const int tid = threadIdx.x, lane = tid & 63;
  if (T <= 0) return 0;
  // first histogram cell (scanning from the best) at which the running count reaches `want`
  auto find_cell = [&](int want, int32_t* cell, int32_t* before) {
    if (tid < 64) {
      int c[4], sum = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) { c[q] = s.scan[4 * lane + q]; sum += c[q]; }
      int incl = sum;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        int x = __shfl_up(incl, o, 64);
        if (lane >= o) incl += x;
      }
      int run = incl - sum, found = -1, bef = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (found < 0 && run + c[q] >= want) { found = 4 * lane + q; bef = run; }
        run += c[q];
      }
      const unsigned long long hit = __builtin_amdgcn_ballot_w64(found >= 0);
      if (hit) {
        const int src = __builtin_ctzll(hit);
        found = __builtin_amdgcn_readlane(found, src);
        bef = __builtin_amdgcn_readlane(bef, src);
      } else {
        found = 256;                                   // fewer than `want` in all cells: everything qualifies
        bef = __builtin_amdgcn_readlane(incl, 63);
      }
      if (lane == 0) { *cell = found; *before = bef; }
    }
  };
  if (tid == 0) { s.n_surv = 0; s.bin1 = 256; s.bin2 = 256; s.before1 = 0; }
  if (n > 256) {
    s.scan[tid] = 0;
    __syncthreads();
    for (int t = tid; t < n; t += 256)
      if (eligible(t)) atomicAdd(&s.scan[(int)(cand_key(s.prob[t], t) >> 55) & 0xff], 1);
    __syncthreads();
    find_cell(T, &s.bin1, &s.before1);
    __syncthreads();
    const int b1 = s.bin1;
    if (b1 < 256) {
      s.scan[tid] = 0;
      __syncthreads();
      for (int t = tid; t < n; t += 256)
        if (eligible(t)) {
          const uint64_t kx = cand_key(s.prob[t], t);
          if (((int)(kx >> 55) & 0xff) == b1) atomicAdd(&s.scan[(int)(kx >> 47) & 0xff], 1);
        }
      __syncthreads();
      int32_t unused_before;
      find_cell(T - s.before1, &s.bin2, tid == 0 ? &s.n_expand : &unused_before);   // n_expand: scratch
    }
  }
  __syncthreads();
  const int b1 = s.bin1, b2 = s.bin2;
  for (int t = tid; t < n; t += 256)
    if (eligible(t)) {
      const uint64_t kx = cand_key(s.prob[t], t);
      const int c1 = (int)(kx >> 55) & 0xff, c2 = (int)(kx >> 47) & 0xff;
      if (c1 < b1 || (c1 == b1 && c2 <= b2)) {
        const int idx = atomicAdd(&s.n_surv, 1);
        if (idx < 256) s.key[idx] = kx;
      }
    }
  __syncthreads();
  const int ns = s.n_surv;
  if (ns > 256) return -1;
  if (tid < ns) {
    const uint64_t kj = s.key[tid];
    int rank = 0;
    for (int i = 0; i < ns; ++i) rank += s.key[i] < kj ? 1 : 0;
    if (rank < T) out[rank] = (int)(kj & 0xffffffffu);
  }
  __syncthreads();
  return min(T, ns);
}

__global__ __launch_bounds__(256) void k_build_tree(esp_tree_params p, const int32_t* __restrict__ topk_id,
                                                    const float* __restrict__ topk_p, int kp,
                                                    const int32_t* __restrict__ n_lists,
                                                    const int32_t* __restrict__ n_emit,
                                                    const int32_t* __restrict__ emit_tok, int rows_per_seq,
                                                    int anc_words, int32_t* n_rows, int32_t* n_nodes, int32_t* tok,
                                                    int32_t* parent, int32_t* depth, int32_t* mask_j,
                                                    int32_t* attach, uint64_t* anc, int32_t* status, int reuse) {
  extern __shared__ __align__(16) unsigned char raw[];
  TreeLds& s = *reinterpret_cast<TreeLds*>(raw);
  __shared__ int s_bad;
  const int seq = blockIdx.x, tid = threadIdx.x;
  const size_t r0 = (size_t)seq * rows_per_seq;
  const int ne = n_emit[seq];
  const bool is_static = p.static_widths[0] > 0;
  int depth_limit = min(p.k, n_lists[seq]);
  if (ne < 1 || ne > ESP_MAX_MASKS + 1) {   // sequence skipped upstream
    if (tid == 0) { n_rows[seq] = 0; n_nodes[seq] = 0; atomicOr(status, ESP_DEV_BAD_TREE); }
    return;
  }
  if (is_static && reuse && depth_limit == p.k) {
    // Fixed tree whose rows this block already holds (Sec. 4.3: the descriptor of a static tree is
    // built once): the shape -- root, K_1 children, K_i children under the first node of depth i - 1
    // -- does not depend on the lists, so parents, depths, mask rows and ancestor sets stay and
    // only the tokens are written.  A thread per node walks the chain of first children down to its
    // own depth.  If a list runs out of surviving entries the shape would change: then (all threads
    // agree first, before anything is written) the full build below runs instead.
    int n_static = 1;
    for (int i = 0; i < p.k; ++i) n_static += p.static_widths[i];
    if (n_nodes[seq] == n_static) {
      const int root = emit_tok[(size_t)seq * (ESP_MAX_MASKS + 1) + ne - 1];
      int my_depth = 0, my_j = 0, base = 1;
      for (int i = 1; i <= p.k; ++i) {
        if (tid >= base && tid < base + p.static_widths[i - 1]) { my_depth = i; my_j = tid - base; }
        base += p.static_widths[i - 1];
      }
      const bool live = tid < n_static;
      int ok = 1, par_tok = root, my_tok = root;
      for (int i = 1; i <= p.k && live && my_depth >= i; ++i) {
        const int32_t* li = topk_id + ((size_t)seq * p.k + (i - 1)) * kp;
        const int want = my_depth == i ? my_j : 0;       // own entry at the own depth, the first child above
        int cnt = 0, pick = -1;
        for (int c = 0; c < kp; ++c) {
          const int t = li[c];
          if (t < 0) break;
          if (p.prune_parent && t == par_tok) continue;
          if (p.prune_last && i >= 2 && t == root) continue;
          if (cnt == want) { pick = t; break; }
          ++cnt;
        }
        if (pick < 0) ok = 0;
        if (my_depth == i) my_tok = pick; else par_tok = pick;
      }
      if (!__syncthreads_or(!ok)) {
        if (live) tok[r0 + tid] = my_tok;
        return;
      }
    }
  }
  if (tid == 0) {
    s.tok[0] = emit_tok[(size_t)seq * (ESP_MAX_MASKS + 1) + ne - 1];
    s.prob[0] = 1.0f;
    s.par[0] = -1;
    s.dep[0] = 0;
    s.used[0] = 1;
    s.n_total = 1;
    s.frontier[0] = 0;
    s.n_frontier = 1;
    s.bad = 0;
  }
  for (int t = tid; t < p.k * kp; t += 256) {
    s.list_id[t] = topk_id[(size_t)seq * p.k * kp + t];
    s.list_p[t] = topk_p[(size_t)seq * p.k * kp + t];
  }
  __syncthreads();
  const int32_t* ids = s.list_id;
  const float* ps = s.list_p;

  for (int i = 1; i <= depth_limit; ++i) {
    // nodes of the current set at depth i-1, in (P desc, creation asc) order, first expand_width
    const int nf = s.n_frontier;
    int flag = (tid < nf && s.dep[s.frontier[tid]] == i - 1) ? 1 : 0;
    int tot;
    int pos = block_excl_scan(flag, s.scan, &tot);
    int n_exp = p.expand_width > 0 ? min(tot, p.expand_width) : tot;
    if (flag && pos < n_exp) s.expand[pos] = s.frontier[tid];
    __syncthreads();
    const int want = is_static ? p.static_widths[i - 1] : min(p.K, p.B - i);
    const int32_t* li = ids + (size_t)(i - 1) * kp;
    const float* lp = ps + (size_t)(i - 1) * kp;
    // children per expanded node: first `want` list entries that survive the pruning rule
    int cnt = 0, node = -1;
    if (tid < n_exp) {
      node = s.expand[tid];
      for (int c = 0; c < kp && cnt < want; ++c) {
        int t = li[c];
        if (t < 0) break;
        if (p.prune_parent && t == s.tok[node]) continue;
        if (p.prune_last && i >= 2 && t == s.tok[0]) continue;
        ++cnt;
      }
    }
    int off = block_excl_scan(cnt, s.scan, &tot);
    const int n_old = s.n_total;
    if (n_old + tot > MAXC) {
      if (tid == 0) s.bad = 1;
      __syncthreads();
      break;
    }
    if (tid < n_exp) {
      int made = 0;
      for (int c = 0; c < kp && made < want; ++c) {
        int t = li[c];
        if (t < 0) break;
        if (p.prune_parent && t == s.tok[node]) continue;
        if (p.prune_last && i >= 2 && t == s.tok[0]) continue;
        int idx = n_old + off + made;
        s.tok[idx] = t;
        s.prob[idx] = s.prob[node] * lp[c];     // one fp32 product (Alg. 1: P(c) = P(n) * P(t|l))
        s.par[idx] = (int16_t)node;
        s.dep[idx] = (uint8_t)i;
        s.used[idx] = 0;
        ++made;
      }
    }
    __syncthreads();
    if (tid == 0) s.n_total = n_old + tot;
    __syncthreads();
    if (i < depth_limit) {
      if (is_static) {
        // fixed tree: the new node set is exactly the fresh children
        for (int t = tid; t < tot && t < ESP_MAX_TREE_NODES; t += 256) s.frontier[t] = n_old + t;
        if (tid == 0) s.n_frontier = min(tot, (int)ESP_MAX_TREE_NODES);
        __syncthreads();
      } else {
        // node set <- the B-i most probable candidates not used before
        const int n = s.n_total;
        const int got = select_best(s, n, max(p.B - i, 0), [&](int t) { return !s.used[t]; }, s.frontier);
        if (got >= 0) {
          if (tid < got) s.used[s.frontier[tid]] = 1;
          if (tid == 0) s.n_frontier = got;
          __syncthreads();
          continue;
        }
        int n2 = 1;
        while (n2 < n) n2 <<= 1;
        for (int t = tid; t < n2; t += 256)
          s.key[t] = (t < n && !s.used[t]) ? cand_key(s.prob[t], t) : ~0ull;
        __syncthreads();
        bitonic_sort(s.key, n2);
        const int take = max(p.B - i, 0);
        for (int t = tid; t < take && t < n2; t += 256) {
          uint64_t kx = s.key[t];
          if (kx != ~0ull) {
            int c = (int)(kx & 0xffffffffu);
            s.frontier[t] = c;
            s.used[c] = 1;
          }
        }
        __syncthreads();
        if (tid == 0) {
          int cntf = 0;
          while (cntf < take && cntf < n2 && s.key[cntf] != ~0ull) ++cntf;
          s.n_frontier = cntf;
        }
        __syncthreads();
      }
    }
  }
  __syncthreads();

  // final selection: root + the B-1 most probable of all candidates (static: all of them)
  const int n = s.n_total;
  int n_keep = n - 1;
  int32_t* kept = s.expand;                 // kept candidates in selection order (free after the loop)
  if (!s.bad) {
    if (!is_static) {
      n_keep = min(n - 1, max(p.B - 1, 0));
      const int got = select_best(s, n, n_keep, [](int t) { return t >= 1; }, kept);
      if (got < 0) {
        int n2 = 1;
        while (n2 < n) n2 <<= 1;
        for (int t = tid; t < n2; t += 256) s.key[t] = (t >= 1 && t < n) ? cand_key(s.prob[t], t) : ~0ull;
        __syncthreads();
        bitonic_sort(s.key, n2);
        if (tid < n_keep) kept[tid] = (int)(s.key[tid] & 0xffffffffu);
      }
    } else if (n_keep + 1 <= ESP_MAX_TREE_NODES) {
      if (tid < n_keep) kept[tid] = tid + 1;              // fixed tree: every candidate, creation order
    }
    if (n_keep + 1 > ESP_MAX_TREE_NODES) {
      if (tid == 0) s.bad = 1;
    }
  }
  __syncthreads();
  if (s.bad) {
    if (tid == 0) { n_rows[seq] = 0; n_nodes[seq] = 0; atomicOr(status, ESP_DEV_BAD_TREE); }
    return;
  }
  // rows: kept nodes ordered by (depth, creation); n_keep <= 255 so one thread per kept node
  int my = -1, my_rank = 0;
  if (tid < n_keep) my = kept[tid];
  __syncthreads();
  if (tid < n_keep) s.scan[tid] = my;
  __syncthreads();
  if (tid < n_keep) {
    uint32_t mk = ((uint32_t)s.dep[my] << 24) | (uint32_t)my;
    for (int u = 0; u < n_keep; ++u) {
      int o = s.scan[u];
      uint32_t ok = ((uint32_t)s.dep[o] << 24) | (uint32_t)o;
      my_rank += ok < mk ? 1 : 0;
    }
  }
  __syncthreads();
  // creation index -> new row, kept in the (now free) sort buffer
  int32_t* new_row = reinterpret_cast<int32_t*>(s.key);
  if (tid == 0) new_row[0] = 0;
  if (tid < n_keep) new_row[my] = my_rank + 1;
  __syncthreads();
  if (tid == 0) {
    tok[r0] = s.tok[0];
    parent[r0] = -1;
    n_nodes[seq] = n_keep + 1;
  }
  if (tid < n_keep) {
    tok[r0 + my_rank + 1] = s.tok[my];
    parent[r0 + my_rank + 1] = new_row[s.par[my]];
  }
  __syncthreads();
  finalize_block(seq, rows_per_seq, p.k, p.layout, anc_words, n_rows, n_keep + 1, tok, parent, depth, mask_j,
                 attach, anc, status, &s_bad);
}

}  // namespace

hipError_t launch_block_from_tree(hipStream_t st, int batch, int rows_per_seq, int k, int layout, int anc_words,
                                  int32_t* n_rows, const int32_t* n_nodes, int32_t* tok, int32_t* parent,
                                  int32_t* depth, int32_t* mask_j, int32_t* attach, uint64_t* anc,
                                  int32_t* status) {
  hipLaunchKernelGGL(k_block_from_tree, dim3(batch), dim3(256), 0, st, rows_per_seq, k, layout, anc_words, n_rows,
                     n_nodes, tok, parent, depth, mask_j, attach, anc, status);
  return hipGetLastError();
}

hipError_t launch_verify_accept(hipStream_t st, int dtype, const BlockDev& b, const KvDev& kv,
                                const int32_t* node_argmax, int n_layers, int n_kv, int hd, int32_t* n_emit,
                                int32_t* emit_tok, int32_t* accepted_row, int32_t* star_row, int32_t* status) {
  (void)status;
  hipLaunchKernelGGL(k_verify, dim3(b.batch), dim3(256), 0, st, b, kv, node_argmax, n_emit, emit_tok,
                     accepted_row, star_row);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid(n_layers * n_kv, b.batch);
  if (dtype == ESP_F32)
    hipLaunchKernelGGL(k_kv_commit<float>, grid, dim3(hd), 0, st, b, kv, n_kv, hd, n_emit, accepted_row);
  else
    hipLaunchKernelGGL(k_kv_commit<bf16_t>, grid, dim3(hd), 0, st, b, kv, n_kv, hd, n_emit, accepted_row);
  return hipGetLastError();
}

hipError_t launch_mask_rows(hipStream_t st, const BlockDev& b, const int32_t* star_row, const int32_t* n_emit,
                            int32_t* a_rows, int32_t* n_lists) {
  hipLaunchKernelGGL(k_mask_rows, dim3(b.batch), dim3(64), 0, st, b, star_row, n_emit, a_rows, n_lists);
  return hipGetLastError();
}

hipError_t launch_build_tree(hipStream_t st, const esp_tree_params& p, int batch, const int32_t* topk_id,
                             const float* topk_p, int kp, const int32_t* n_lists, const int32_t* n_emit,
                             const int32_t* emit_tok, int rows_per_seq, int anc_words, int32_t* n_rows,
                             int32_t* n_nodes, int32_t* tok, int32_t* parent, int32_t* depth, int32_t* mask_j,
                             int32_t* attach, uint64_t* anc, int32_t* status, bool reuse) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_build_tree),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(TreeLds));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(k_build_tree, dim3(batch), dim3(256), sizeof(TreeLds), st, p, topk_id, topk_p, kp, n_lists,
                     n_emit, emit_tok, rows_per_seq, anc_words, n_rows, n_nodes, tok, parent, depth, mask_j,
                     attach, anc, status, reuse ? 1 : 0);
  return hipGetLastError();
}
