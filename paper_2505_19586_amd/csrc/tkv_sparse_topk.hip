// tkv_sparse_estimate_topk: Stage 2 of the dynamic retrieval (Sec. 4.2): approximate
// scores of every cached token from the critical query channels and the critical key
// cache, then exact Top-K (ties to the lower token index, output ascending).
//
// Three launches, each fully parallel (the histogram and counters in the workspace must
// be zero before the first call; every call leaves them zero):
//   score    reads the key summary once, computes S(t) in the pinned float32 order, writes
//            an order-preserving 32-bit key per token and a 13-bit-prefix histogram; the
//            last workgroup of a head locates the histogram bin that holds the k-th key;
//   filter   counts, per 1024-token block, the keys above that bin and appends the keys
//            inside it (a few hundred) to a candidate list;
//   finish   every block finds the exact threshold among the candidates (radix select on
//            the remaining 19 key bits), then writes its own selected tokens at the right
//            offset, in token order.
#include "tkv_common.h"

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kTok = 4096;      // tokens per workgroup (256 threads x 16)
constexpr int kBatch = 4;       // tokens a thread has in flight at once
constexpr int kPrefixBits = 13;
constexpr int kBins = 1 << kPrefixBits;  // 8192
constexpr int kLowBits = 32 - kPrefixBits;  // 19
constexpr uint32_t kLowMask = (1u << kLowBits) - 1u;

enum Ctrl { kDone = 0, kNCand = 1, kBin = 2, kAbove = 3, kCtrlWords = 8 };

struct TopkParams {
  const __half* summary;
  const int32_t* channel_idx;
  const __half* q;
  int32_t* topk_idx;
  int32_t* topk_count;
  tkv::SparseWs ws;
  int32_t hq, hkv, top_k, n_sink, n_window, capacity;
  TkvSeqLens lens;
};

// Larger float <-> larger unsigned key; +0 and -0 were already merged by "+ 0.0f".
__device__ inline uint32_t score_key(float s) {
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline void candidate_range(const TopkParams& p, int n, int& lo, int& hi) {
  lo = min(p.n_sink, n);
  hi = max(n - p.n_window, lo);
}

__device__ inline uint32_t k_eff_of(const TopkParams& p, int n) {
  int lo, hi;
  candidate_range(p, n, lo, hi);
  return (uint32_t)min(p.top_k, hi - lo);
}

// Inclusive suffix sums over the 256 threads of a workgroup: returns sum of v over
// threads >= tid.  scratch holds 8 words.
__device__ inline uint32_t block_suffix_sum(uint32_t v, uint32_t* scratch) {
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  uint32_t s = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t o = __shfl_down(s, d, 64);
    if (lane + d < 64) s += o;
  }
  if (lane == 0) scratch[wave] = s;  // wave totals
  __syncthreads();
  for (int w = wave + 1; w < 4; ++w) s += scratch[w];
  __syncthreads();
  return s;
}

// Finds, in a histogram of `nbins` (multiple of 256) counts where larger bin = larger
// key, the bin that holds the k-th largest key: `above` keys lie in higher bins,
// above < k <= above + count[bin].  Result valid in every thread.
__device__ inline void find_bin(const uint32_t* hist, int nbins, uint32_t k, uint32_t* scratch /*>= 10 words*/,
                                uint32_t& bin, uint32_t& above) {
  const int tid = threadIdx.x;
  const int per = nbins / 256;
  uint32_t local = 0;
  for (int i = 0; i < per; ++i) local += hist[tid * per + i];
  const uint32_t incl = block_suffix_sum(local, scratch);  // keys in this thread's bins and higher
  const uint32_t excl = incl - local;
  if (excl < k && k <= incl) {  // exactly one thread
    uint32_t run = excl;
    int bsel = tid * per + per - 1;
    for (; bsel > tid * per; --bsel) {
      const uint32_t c = hist[bsel];
      if (run + c >= k) break;
      run += c;
    }
    scratch[8] = (uint32_t)bsel;
    scratch[9] = run;
  }
  __syncthreads();
  bin = scratch[8];
  above = scratch[9];
  __syncthreads();
}

__device__ inline void reset_head(uint32_t* gh, uint32_t* ctrl);

// score + key + histogram; the last workgroup of each head resolves the bin and clears
// the histogram and counters for the next call.
template <int DS>
__global__ __launch_bounds__(256) void score_kernel(TopkParams p) {
  __shared__ uint32_t hist[kBins];
  __shared__ float qc[4][DS];
  __shared__ uint32_t scratch[12];
  const int b = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const int n = p.lens.n[b];
  const int t0 = blockIdx.x * kTok;
  if (t0 >= n) return;
  int lo, hi;
  candidate_range(p, n, lo, hi);
  const uint32_t k = (uint32_t)min(p.top_k, hi - lo);
  const int G = p.hq / p.hkv;
  const size_t bh = (size_t)b * p.hkv + h;
  for (int i = tid; i < kBins; i += 256) hist[i] = 0u;
  if (tid < 4 * DS) {
    const int j = tid / DS, i = tid % DS;
    const int c = p.channel_idx[bh * DS + i];
    qc[j][i] = j < G ? __half2float(p.q[((size_t)b * p.hq + (size_t)h * G + j) * TKV_D + c]) : 0.f;
  }
  __syncthreads();

  // query channels into registers (heads >= G are zero: adding their +0 sums changes nothing)
  float qr[4][DS];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < DS; ++i) qr[j][i] = qc[j][i];

  const __half* srow = p.summary + (bh * p.capacity) * DS;
  uint32_t* keys = p.ws.keys + bh * p.capacity;
  // Batches of 4 tokens per thread; the next batch's loads (clamped to the last token) are
  // in flight while the current batch is scored.
  typedef uint4 RowBatch[kBatch][DS / 8];
  auto load_batch = [&](RowBatch& rows, int bt) {
    const int tb0 = t0 + bt * kBatch * 256;
#pragma unroll
    for (int it = 0; it < kBatch; ++it) {
      const int t = min(tb0 + it * 256 + tid, n - 1);
#pragma unroll
      for (int x = 0; x < DS / 8; ++x) rows[it][x] = reinterpret_cast<const uint4*>(srow + (size_t)t * DS)[x];
    }
  };
  auto score_batch = [&](const RowBatch& rows, int bt) {
    const int tb0 = t0 + bt * kBatch * 256;
#pragma unroll
    for (int it = 0; it < kBatch; ++it) {
      const int t = tb0 + it * 256 + tid;
      float kx[DS];
#pragma unroll
      for (int x = 0; x < DS / 8; ++x) {
        const uint32_t w[4] = {rows[it][x].x, rows[it][x].y, rows[it][x].z, rows[it][x].w};
#pragma unroll
        for (int y = 0; y < 4; ++y) {
          const uint32_t wy = w[y];
          const half2_t hh = __builtin_bit_cast(half2_t, wy);
          kx[8 * x + 2 * y] = (float)hh[0];
          kx[8 * x + 2 * y + 1] = (float)hh[1];
        }
      }
      float total = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // left-to-right sum of exact products: fma(q, k, a) rounds once, like a + q*k
        float a = qr[j][0] * kx[0];
#pragma unroll
        for (int i = 1; i < DS; ++i) a = __builtin_fmaf(qr[j][i], kx[i], a);
        total = j == 0 ? a : total + a;
      }
      total = total + 0.0f;
      if (t < n) {
        uint32_t key = 0u;  // non-candidates: below every finite score
        if (t >= lo && t < hi) {
          key = score_key(total);
          atomicAdd(&hist[key >> kLowBits], 1u);
        }
        keys[t] = key;
      }
    }
  };
  static_assert(kTok / (256 * kBatch) == 4, "four batches per workgroup");
  {
    RowBatch ra, rb;
    load_batch(ra, 0);
    load_batch(rb, 1);
    score_batch(ra, 0);
    load_batch(ra, 2);
    score_batch(rb, 1);
    load_batch(rb, 3);
    score_batch(ra, 2);
    score_batch(rb, 3);
  }
  __syncthreads();
  // Only bins that can hold the head's k-th key go to the global histogram: the k-th key of
  // the whole head is never below the k-th key of this block alone, so bins under the
  // block's own k-th bin are irrelevant (and skipping them spares most global atomics).
  uint32_t first_bin = 0;
  {
    const int c_lo = max(lo, t0), c_hi = min(hi, min(n, t0 + kTok));
    if (c_hi - c_lo >= (int)k && k > 0) {
      uint32_t above_unused;
      find_bin(hist, kBins, k, scratch, first_bin, above_unused);
    }
  }
  __syncthreads();
  uint32_t* gh = p.ws.hist + bh * kBins;
  uint32_t* ctrl = p.ws.ctrl + bh * kCtrlWords;
  for (int i = tid; i < kBins; i += 256)
    if (i >= (int)first_bin && hist[i]) atomicAdd(&gh[i], hist[i]);
  // Last workgroup of this head: locate the bin of the k-th key.  The histogram is only
  // touched with device-scope atomics, which are coherent by themselves: waiting for this
  // wave's atomics to complete orders them before the arrival counter without a cache
  // write-back (a release fence would flush the keys just written from L2).
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) {
    const uint32_t nblk = (uint32_t)((n + kTok - 1) / kTok);
    scratch[11] = atomicAdd(&ctrl[kDone], 1u) == nblk - 1u;
  }
  __syncthreads();
  if (!scratch[11]) return;
  // the head's bin is never below this block's own first_bin: lower bins are not needed
  for (int i = tid; i < kBins; i += 256)
    hist[i] = i >= (int)first_bin ? __atomic_load_n(&gh[i], __ATOMIC_RELAXED) : 0u;
  __syncthreads();
  reset_head(gh, ctrl);
  if (k == 0) return;
  uint32_t bin, above;
  find_bin(hist, kBins, k, scratch, bin, above);
  if (tid == 0) {
    ctrl[kBin] = bin;
    ctrl[kAbove] = above;
  }
}

// Leaves the histogram and counters of one head zero again for the next call.
__device__ inline void reset_head(uint32_t* gh, uint32_t* ctrl) {
  for (int i = threadIdx.x; i < kBins; i += 256) gh[i] = 0u;
  if (threadIdx.x == 0) {
    ctrl[kDone] = 0u;
    ctrl[kNCand] = 0u;
  }
}

__global__ __launch_bounds__(256) void filter_kernel(TopkParams p) {
  __shared__ uint32_t s_gt, s_nc, s_base;
  __shared__ uint2 s_cand[kTok];
  const int b = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const int n = p.lens.n[b];
  const int t0 = blockIdx.x * kTok;
  if (t0 >= n) return;
  if (k_eff_of(p, n) == 0) return;
  const size_t bh = (size_t)b * p.hkv + h;
  uint32_t* ctrl = p.ws.ctrl + bh * kCtrlWords;
  const uint32_t bin = ctrl[kBin];
  if (tid == 0) {
    s_gt = 0u;
    s_nc = 0u;
  }
  __syncthreads();
  const uint32_t* keys = p.ws.keys + bh * p.capacity;
  uint32_t gt = 0;
  for (int i = tid; i < kTok; i += 256) {
    const int t = t0 + i;
    if (t >= n) break;
    const uint32_t key = keys[t];
    if (key != 0u) {
      const uint32_t pre = key >> kLowBits;
      gt += pre > bin;
      if (pre == bin) s_cand[atomicAdd(&s_nc, 1u)] = make_uint2(key, (uint32_t)t);
    }
  }
  for (int m = 32; m >= 1; m >>= 1) gt += __shfl_xor(gt, m, 64);
  if (tid % 64 == 0 && gt) atomicAdd(&s_gt, gt);
  __syncthreads();
  // one global reservation per block for its candidates
  if (tid == 0) {
    p.ws.blk[bh * p.ws.nblk_cap + blockIdx.x] = s_gt;
    s_base = s_nc ? atomicAdd(&ctrl[kNCand], s_nc) : 0u;
  }
  __syncthreads();
  uint2* cand = p.ws.cand + bh * (size_t)p.capacity + s_base;
  for (uint32_t i = tid; i < s_nc; i += 256) cand[i] = s_cand[i];
}

__global__ __launch_bounds__(256) void finish_kernel(TopkParams p) {
  __shared__ uint32_t hist[1024];
  __shared__ uint32_t scratch[12];
  __shared__ uint32_t sgt[256], seq[256];
  const int b = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const int n = p.lens.n[b];
  const size_t bh = (size_t)b * p.hkv + h;
  const uint32_t k = k_eff_of(p, n);
  int32_t* out = p.topk_idx + bh * p.top_k;
  if (blockIdx.x == 0) {
    for (int i = (int)k + tid; i < p.top_k; i += 256) out[i] = -1;
    if (tid == 0) p.topk_count[bh] = (int32_t)k;
  }
  const int t0 = blockIdx.x * kTok;
  if (t0 >= n || k == 0) return;
  const uint32_t* ctrl = p.ws.ctrl + bh * kCtrlWords;
  const uint32_t bin = ctrl[kBin], above = ctrl[kAbove], ncand = ctrl[kNCand];
  const uint2* cand = p.ws.cand + bh * (size_t)p.capacity;
  uint32_t k_rem = k - above;  // 1 <= k_rem <= ncand

  // exact threshold inside the bin: radix select on the low 19 key bits (10 + 9)
  for (int i = tid; i < 1024; i += 256) hist[i] = 0u;
  __syncthreads();
  for (uint32_t i = tid; i < ncand; i += 256) atomicAdd(&hist[(cand[i].x & kLowMask) >> 9], 1u);
  __syncthreads();
  uint32_t d1, a1;
  find_bin(hist, 1024, k_rem, scratch, d1, a1);
  k_rem -= a1;
  for (int i = tid; i < 1024; i += 256) hist[i] = 0u;
  __syncthreads();
  for (uint32_t i = tid; i < ncand; i += 256) {
    const uint32_t low = cand[i].x & kLowMask;
    if ((low >> 9) == d1) atomicAdd(&hist[low & 0x1FFu], 1u);
  }
  __syncthreads();
  uint32_t d2, a2;
  find_bin(hist, 512, k_rem, scratch, d2, a2);
  const uint32_t take = k_rem - a2;                       // keys equal to T that are selected (lowest indices)
  const uint32_t T = (bin << kLowBits) | (d1 << 9) | d2;  // threshold key

  // selected keys in earlier blocks: above the bin (per-block counts), inside the bin
  // above T, and equal to T (candidates are few; every block scans them)
  uint32_t gt_before = 0, eq_before = 0;
  for (int i = tid; i < (int)blockIdx.x; i += 256) gt_before += p.ws.blk[bh * p.ws.nblk_cap + i];
  for (uint32_t i = tid; i < ncand; i += 256) {
    const uint2 c = cand[i];
    if ((int)c.y < t0) {
      gt_before += c.x > T;
      eq_before += c.x == T;
    }
  }
  sgt[tid] = gt_before;
  seq[tid] = eq_before;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) {
      sgt[tid] += sgt[tid + s];
      seq[tid] += seq[tid + s];
    }
    __syncthreads();
  }
  gt_before = sgt[0];
  eq_before = seq[0];
  __syncthreads();

  // ordered compaction of this block's tokens: thread i owns tokens t0 + 16 i .. + 15
  constexpr int PT = kTok / 256;
  const uint32_t* keys = p.ws.keys + bh * p.capacity;
  uint32_t key[PT];
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int x = 0; x < PT; ++x) {
    const int t = t0 + PT * tid + x;
    key[x] = t < n ? keys[t] : 0u;
    gt += key[x] > T;
    eq += key[x] == T && key[x] != 0u;
  }
  sgt[tid] = gt;
  seq[tid] = eq;
  __syncthreads();
  for (int s = 1; s < 256; s <<= 1) {  // inclusive scan over threads
    uint32_t a = 0, c = 0;
    if (tid >= s) {
      a = sgt[tid - s];
      c = seq[tid - s];
    }
    __syncthreads();
    sgt[tid] += a;
    seq[tid] += c;
    __syncthreads();
  }
  uint32_t gt_run = gt_before + sgt[tid] - gt;
  uint32_t eq_run = eq_before + seq[tid] - eq;
  if (gt + eq) {
#pragma unroll
    for (int x = 0; x < PT; ++x) {
      const int t = t0 + PT * tid + x;
      if (key[x] > T) {
        out[gt_run + min(eq_run, take)] = t;
        ++gt_run;
      } else if (key[x] == T && key[x] != 0u) {
        if (eq_run < take) out[gt_run + eq_run] = t;
        ++eq_run;
      }
    }
  }
}

}  // namespace

extern "C" int32_t tkv_sparse_estimate_topk(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const void* q,
                                            int32_t* topk_idx, int32_t* topk_count, void* workspace,
                                            size_t workspace_bytes, void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !c->key_summary || !c->channel_idx || !q || !topk_idx || !topk_count || !workspace)
    return TKV_E_INVAL;
  size_t need = 0;
  tkv_sparse_cache_sizes(d, nullptr, &need);
  if (workspace_bytes < need) return TKV_E_WORKSPACE;
  TopkParams p;
  int max_n = 0;
  for (int b = 0; b < d->batch; ++b) {
    const int32_t n = c->seq_len_host[b];
    if (n < 0) return TKV_E_INVAL;
    if (n > d->capacity) return TKV_E_CAPACITY;
    p.lens.n[b] = n;
    if (n > max_n) max_n = n;
  }
  p.summary = (const __half*)c->key_summary;
  p.channel_idx = c->channel_idx;
  p.q = (const __half*)q;
  p.topk_idx = topk_idx;
  p.topk_count = topk_count;
  p.ws = tkv::carve_sparse_ws(d, workspace);
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.top_k = d->top_k;
  p.n_sink = d->n_sink;
  p.n_window = d->n_window;
  p.capacity = d->capacity;

  hipStream_t s = (hipStream_t)stream;
  int nblk = (max_n + kTok - 1) / kTok;
  if (nblk < 1) nblk = 1;
  const dim3 grid(nblk, d->n_kv_heads, d->batch);
  if (d->n_channels == 16)
    score_kernel<16><<<grid, 256, 0, s>>>(p);
  else
    score_kernel<8><<<grid, 256, 0, s>>>(p);
  filter_kernel<<<grid, 256, 0, s>>>(p);
  finish_kernel<<<grid, 256, 0, s>>>(p);
  return tkv::launch_status();
}
