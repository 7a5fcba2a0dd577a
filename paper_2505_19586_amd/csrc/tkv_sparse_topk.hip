// tkv_sparse_estimate_topk: Stage 2 of the dynamic retrieval (Sec. 4.2): approximate
// scores of every cached token from the critical query channels and the critical key
// cache, then exact Top-K (ties to the lower token index, output ascending).
//
// One launch.  A workgroup owns a contiguous share of a head's tokens (the entry point sizes
// the shares so that the workgroups fill the machine a whole number of times) and scores it:
// the critical key cache is read once (token-major summary, or channel-major rows), S(t) is
// computed in the pinned float32 order and kept in registers as an order-preserving 32-bit
// key, together with an LDS histogram of the keys' 13-bit prefix ("bin").  No key and no
// histogram is ever written to memory.  Then
//   * the workgroup lists, in token order, its tokens at or above a bin L of its own choice:
//     the bin of its r-th largest key, r = 1.5 x its fair share of k plus 16.  If the head's
//     Top-K were spread evenly, every workgroup would hold its fair share of it, so L almost
//     always lies at or below the bin of the head's k-th key and the list holds every token of
//     this workgroup that can be selected.  List, list length and L go to the workspace;
//   * the last workgroup of the head to arrive (arrival counter) fetches all lists in one
//     round of device-scope loads (a few thousand entries, held in registers), finds the k-th
//     largest listed key T by radix select and checks that no list's L lies above T's bin:
//     every list is complete down to its L, so T is then the head's exact k-th key.  It writes
//     the tokens above T, and the lowest-numbered ones equal to T, in token order;
//   * otherwise (some workgroup's tokens hold far more than their share of the Top-K, or lists
//     longer than the round fetches: heavy ties) the last workgroup takes the slow path: lists
//     concatenated in LDS, T from them, the workgroups whose L lies above T's bin re-scored and
//     listed again down to that bin, T again: more entries can only raise T, so every list is
//     now complete down to a bin at or below T's.  The result never depends on the guess, only
//     the time does.
// Optional riders of the launch: Eq. 10's channel selection at the start of every workgroup
// (resident channel-major keys), and the decode step's cache update (Eq. 2) by one more
// workgroup per head.  The counters in the workspace must be zero before the first call; every
// call leaves them zero.
// Inside a launch, data crosses workgroups only through device-scope stores, loads and
// atomics, ordered by waiting for them to complete before an arrival counter is bumped.
#include <type_traits>

#include "tkv_common.h"

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kThreads = 1024;
constexpr int kWavesPerBlock = kThreads / 64;
constexpr int kPer = 4;                // tokens per thread in the scoring phase
constexpr int kTok = kThreads * kPer;  // tokens per workgroup and pass
constexpr int kSub = kPer + 1;         // sub-tiles of kThreads tokens per workgroup: a full pass and one more sub-tile
constexpr int kMaxTpw = kSub * kThreads;  // most tokens a workgroup owns (see the entry point)
constexpr int kPrefixBits = 13;
constexpr int kBins = 1 << kPrefixBits;  // 8192
constexpr int kLowBits = 32 - kPrefixBits;  // 19
constexpr int kListCap = 8192;  // candidate entries kept in LDS; further ones go to the workspace
// fused kernel: local / head histogram, list offsets, list (the channel-major variant also
// stages its keys there to put them into token order)
constexpr int kFusedLds = kBins * 4 + 1024 * 4 + kListCap * 8;
constexpr int kFastShift = 14;  // first radix digit of the common path: key bits [14, 32) minus a base
constexpr int kCountBits = 14;  // a workgroup's list length (<= kMaxTpw) in its control word, L above it
static_assert(kMaxTpw < (1 << kCountBits), "list length field");

enum Ctrl { kDone2 = 1, kCtrlWords = 8 };

struct TopkParams {
  const __half* summary;       // token-major [B][Hkv][capacity][d_s], or channel-major rows (below)
  int32_t rows_per_head;       // channel-major: [B][Hkv][rows_per_head][capacity], d_s or 128 rows
  const int32_t* channel_idx;
  const float* k_absmax;       // non-null: Stage 1 in the same launch (Eq. 10 from q_hat and these maxima);
  const __half* q_hat;         //   the list is also written to channel_out
  int32_t* channel_out;
  const __half* q;
  int32_t* topk_idx;
  int32_t* topk_count;
  tkv::SparseWs ws;
  int32_t hq, hkv, top_k, n_sink, n_window, capacity;
  int32_t tpw;  // tokens per workgroup: a multiple of 16, at most kMaxTpw
  TkvSeqLens lens;
  // Eq. 2 in the same launch (app_k non-null): one workgroup of every (sequence, KV head), the
  // first to have handed in its list, appends the step's new tokens; lens already counts them
  const __half* app_k;
  const __half* app_v;
  __half* app_host;     // device-visible view of the pinned host cache
  __half* app_local;
  __half* app_summary;
  int32_t app_stride;   // rows per sequence in app_k / app_v
  TkvSeqLens app_add;
  // Exact attention by the head's last workgroup in the same launch (ATT kernels only)
  const __half* att_host;   // device-visible view of the pinned host cache
  const __half* att_local;
  __half* att_out;          // [B][Hq][D]
  float att_scale2;         // sm_scale * log2(e)
  // (ATT kernels) the key summary that the stream's next call will sweep, same layout as
  // `summary`: read once by the workgroups that are through with the selection while the
  // heads' last workgroups are busy with the host link
  const __half* pf;
  // (ATT kernels) non-zero: topk_idx / topk_count are INPUTS, the selection of an earlier call;
  // the launch (one workgroup per sequence and KV head) only fetches the rows and attends
  int32_t given;
#ifdef TKV_PHASE
  long long* prof;
#endif
};
#ifdef TKV_PHASE
#define TKV_PH(i) do { __builtin_amdgcn_sched_barrier(0); if (p.prof && tid == 0) p.prof[(blockIdx.y * gridDim.x + blockIdx.x) * 32 + (i)] = wall_clock64(); __builtin_amdgcn_sched_barrier(0); } while (0)
#define TKV_PHW(i) do { __builtin_amdgcn_sched_barrier(0); if (p.prof && lane == 0) p.prof[(blockIdx.y * gridDim.x + blockIdx.x) * 32 + (i)] = wall_clock64(); __builtin_amdgcn_sched_barrier(0); } while (0)
#else
#define TKV_PH(i) do {} while (0)
#define TKV_PHW(i) do {} while (0)
#endif

// Larger float <-> larger unsigned key; +0 and -0 were already merged by "+ 0.0f".
__device__ inline uint32_t score_key(float s) {
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline void candidate_range(const TopkParams& p, int n, int& lo, int& hi) {
  lo = min(p.n_sink, n);
  hi = max(n - p.n_window, lo);
}

__device__ inline uint32_t ld_agent(const uint32_t* ptr) {
  return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_agent(uint32_t* ptr, uint32_t v) {
  __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// number of set bits of a wave mask below this lane
__device__ inline uint32_t rank_in(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Inclusive prefix sum over the lanes of a wave (lane l gets the sum of lanes 0..l), on the
// data-parallel-primitive cross-lane paths (no LDS traffic).
#define TKV_DPP_ADD(v, ctrl, rows) \
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(v), ctrl, rows, 0xF, true)
__device__ inline uint32_t wave_prefix_incl(uint32_t v) {
  TKV_DPP_ADD(v, 0x111, 0xF);  // row_shr:1
  TKV_DPP_ADD(v, 0x112, 0xF);  // row_shr:2
  TKV_DPP_ADD(v, 0x114, 0xF);  // row_shr:4
  TKV_DPP_ADD(v, 0x118, 0xF);  // row_shr:8
  TKV_DPP_ADD(v, 0x142, 0xA);  // row_bcast:15 into rows 1 and 3
  TKV_DPP_ADD(v, 0x143, 0xC);  // row_bcast:31 into rows 2 and 3
  return v;
}
#undef TKV_DPP_ADD
// Value of the lane whose number differs in bit D (D = 1 .. 16, within a half-wave of 32): one
// LDS-crossbar swizzle, no address arithmetic.
template <int D>
__device__ inline float swap_xor(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), (D << 10) | 0x1F));
}
__device__ inline uint32_t read_lane(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }

// Finds the bins that hold given ranks of the keys (rank r: the r-th largest), from bin counts
// held in registers: thread t owns the PER bins PER * kThreads - 1 -
// (PER * t + i), i = 0 .. PER - 1 (descending keys), count c[i].  Up to NR ranks at once (rank
// 0: skipped, result bin 0).  res: 2 * NR words of LDS that receive (bin, keys in higher bins)
// per rank; wtot: kWavesPerBlock words of LDS.  Two barriers; results valid in every thread.
template <int NR, int PER>
__device__ inline void find_ranks(const uint32_t (&c)[PER], const uint32_t (&k)[NR], uint32_t* wtot, uint32_t* res,
                                  int wave, int lane) {
  const int tid = threadIdx.x;
  uint32_t local = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) local += c[i];
  const uint32_t incl = wave_prefix_incl(local);
  if (lane == 63) wtot[wave] = incl;
  if (tid < 2 * NR) res[tid] = 0u;
  __syncthreads();
  uint32_t base = 0;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) base += w < wave ? wtot[w] : 0u;
  const uint32_t excl = base + incl - local;  // keys in bins above this thread's
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    if (k[r] != 0u && excl < k[r] && k[r] <= excl + local) {  // exactly one thread per rank
      uint32_t run = excl;
      int i = 0;
#pragma unroll
      for (int y = 0; y < PER - 1; ++y) {
        if (i == y && run + c[y] < k[r]) {
          run += c[y];
          i = y + 1;
        }
      }
      res[2 * r] = (uint32_t)(PER * kThreads - 1 - (PER * tid + i));
      res[2 * r + 1] = run;
    }
  }
  __syncthreads();
}

// Exclusive offsets, in (sub-tile, thread) order, of the set bits of kSub wave ballots per wave:
// before[j] = set bits of sub-tiles < j plus those of sub-tile j in lower waves.  cnt: kSub x
// kWavesPerBlock words of LDS that no thread still reads.  One barrier.  Returns the total.
static_assert(kSub * kWavesPerBlock <= 128, "two count words per lane");
__device__ inline uint32_t subtile_offsets(const unsigned long long (&mask)[kSub], uint32_t* cnt, int wave, int lane,
                                           uint32_t (&before)[kSub]) {
  constexpr int kFlat = kSub * kWavesPerBlock;
  if (lane == 0) {
#pragma unroll
    for (int j = 0; j < kSub; ++j) cnt[j * kWavesPerBlock + wave] = (uint32_t)__builtin_popcountll(mask[j]);
  }
  __syncthreads();
  const uint32_t v0 = cnt[lane], v1 = 64 + lane < kFlat ? cnt[64 + lane] : 0u;
  const uint32_t p0 = wave_prefix_incl(v0), p1 = wave_prefix_incl(v1);
  const uint32_t t0 = read_lane(p0, 63);
  const uint32_t e0 = p0 - v0, e1 = p1 - v1 + t0;
#pragma unroll
  for (int j = 0; j < kSub; ++j)
    before[j] = j < 4 ? read_lane(e0, j * kWavesPerBlock + wave) : read_lane(e1, (j - 4) * kWavesPerBlock + wave);
  return t0 + read_lane(p1, 63);
}

// subtile_offsets for two sets of ballots with one barrier.
__device__ inline void subtile_offsets2(const unsigned long long (&ma)[kSub], const unsigned long long (&mb)[kSub],
                                        uint32_t* cnt_a, uint32_t* cnt_b, int wave, int lane,
                                        uint32_t (&before_a)[kSub], uint32_t (&before_b)[kSub]) {
  constexpr int kFlat = kSub * kWavesPerBlock;
  if (lane == 0) {
#pragma unroll
    for (int j = 0; j < kSub; ++j) {
      cnt_a[j * kWavesPerBlock + wave] = (uint32_t)__builtin_popcountll(ma[j]);
      cnt_b[j * kWavesPerBlock + wave] = (uint32_t)__builtin_popcountll(mb[j]);
    }
  }
  __syncthreads();
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const uint32_t* cnt = which ? cnt_b : cnt_a;
    const uint32_t v0 = cnt[lane], v1 = 64 + lane < kFlat ? cnt[64 + lane] : 0u;
    const uint32_t p0 = wave_prefix_incl(v0), p1 = wave_prefix_incl(v1);
    const uint32_t e0 = p0 - v0, e1 = p1 - v1 + read_lane(p0, 63);
#pragma unroll
    for (int j = 0; j < kSub; ++j) {
      const uint32_t v = j < 4 ? read_lane(e0, j * kWavesPerBlock + wave) : read_lane(e1, (j - 4) * kWavesPerBlock + wave);
      if (which) before_b[j] = v; else before_a[j] = v;
    }
  }
}

// Cache update (Eq. 2) of one KV head by one workgroup: host rows, resident sink / window rows,
// critical channels of the key summary.
template <int DS>
__device__ inline void append_tokens(const TopkParams& p, int b, int h, int tid) {
  const size_t bh = (size_t)b * p.hkv + h;
  const int add = p.app_add.n[b], n1 = p.lens.n[b], n0 = n1 - add;
  for (int x = tid; x < add * 32; x += kThreads) {
    const int i = x / 32, kv = (x % 32) / 16, part = x % 16;
    const int tok = n0 + i;
    const uint4 v = reinterpret_cast<const uint4*>((kv ? p.app_v : p.app_k) +
                                                   (((size_t)b * p.app_stride + i) * p.hkv + h) * TKV_D)[part];
    reinterpret_cast<uint4*>(p.app_host + ((bh * p.capacity + tok) * 2 + kv) * TKV_D)[part] = v;
    const bool local = tok < p.n_sink || tok >= n1 - p.n_window;
    const int slot = tok < p.n_sink ? tok : p.n_sink + tok % p.n_window;
    if (local)
      reinterpret_cast<uint4*>(p.app_local + ((bh * (p.n_sink + p.n_window) + slot) * 2 + kv) * TKV_D)[part] = v;
  }
  for (int x = tid; x < add * DS; x += kThreads) {
    const int i = x / DS, ci = x % DS;
    const int c = p.channel_idx[bh * DS + ci];
    p.app_summary[(bh * p.capacity + (size_t)(n0 + i)) * DS + ci] =
        p.app_k[(((size_t)b * p.app_stride + i) * p.hkv + h) * TKV_D + c];
  }
}

// CM: the critical key cache is channel-major (one row of `capacity` tokens per channel):
// a thread then scores four consecutive tokens, one 8-byte load per channel row.
// GH: query heads per KV head the scores are summed over: 4 (groups of up to 4; their channels
// sit in registers), or 8 (groups of 5 to 8: read from LDS term by term; no ATT form).
template <int DS, bool CM, bool ATT, int GH = 4>
__global__ __launch_bounds__(kThreads) void score_select_kernel(TopkParams p) {
  static_assert(GH == 4 || (GH == 8 && !ATT), "the attention phase holds four heads per lane");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem);                            // kBins words
  uint32_t* offs = reinterpret_cast<uint32_t*>(smem + kBins * 4);                // 1024 words
  uint2* list_s = reinterpret_cast<uint2*>(smem + kBins * 4 + 1024 * 4);         // kListCap entries
  uint32_t* stage = reinterpret_cast<uint32_t*>(list_s);                         // CM: 2 * kTok keys
  __shared__ float qc[GH][DS];
  __shared__ uint32_t scratch[kWavesPerBlock + 8];
  __shared__ uint32_t s_cnt[kSub][kWavesPerBlock], s_cnt2[kSub][kWavesPerBlock];
  __shared__ uint32_t s_wtot[kWavesPerBlock], s_res[2];
  __shared__ uint32_t s_nrep;
  __shared__ uint16_t s_rep[kThreads];
  const int b = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const int lane = tid % 64, wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int n = p.lens.n[b];
  const size_t bh = (size_t)b * p.hkv + h;
  // The step's new tokens (if any) are appended by one workgroup of the head once it has nothing
  // else left to do: the head's first workgroup to arrive, which then only waits for the others
  // (a workgroup of its own would take a compute unit that a scoring workgroup then waits for,
  // the grid being one workgroup per compute unit).  The new tokens are newer than every Top-K
  // candidate (at most n_window of them): the scoring workgroups read their summary rows at most
  // to discard the result, and the attention takes their rows from the call's arguments.
  bool appends = false;
  int32_t* out = p.topk_idx + bh * p.top_k;
  int lo, hi;
  candidate_range(p, n, lo, hi);
  const uint32_t k = (uint32_t)min(p.top_k, hi - lo);
  const int G = p.hq / p.hkv;
  int32_t* sel_s = reinterpret_cast<int32_t*>(smem);  // ATT: the selected tokens (the histogram is no longer needed by then)
  // ---- exact attention (Eq. 3) over sinks + selected + window by this workgroup (ATT only):
  // fetch of the selected rows from the pinned host cache (the transfer that cannot be hidden,
  // Sec. 4.2) and attention in the launch that selected them.  A wave takes 4 attended tokens
  // per pass and has the next two passes on their way: one load instruction per 512-byte row
  // (lanes 0..31 its K half, lanes 32..63 its V half: the request shape the host link serves
  // fastest), the 4 x 4 logits are partial sums of 4 channels per lane, reduced over the 32 key
  // lanes by a butterfly that halves the number of values with every exchange; online softmax
  // per wave, the waves' results meet in LDS.  Rows of the step's new tokens come from the
  // call's k_new / v_new (another workgroup writes them to the cache meanwhile), everything else
  // that is resident from kv_local.  sel: the selected tokens in LDS (ascending), cnt of them.
  auto attend = [&](const int32_t* sel, int cnt) {
    constexpr int R = 4;  // rows per wave and pass
    float* xs = reinterpret_cast<float*>(smem + kBins * 4) + wave * (R * 4);                   // [R][4] logits of this wave
    float* mrg = reinterpret_cast<float*>(smem + kBins * 4 + 1024 * 4);                         // [waves][4][TKV_D + 4]
    const int n_sk = min(p.n_sink, n), w0 = max(n - p.n_window, n_sk);
    // order of the attended tokens: sinks, window, selected -- the resident rows first, worked on
    // while the first host rows are on their way
    const int n_res = n_sk + (n - w0);
    const int n_att = n_res + cnt;
    const int n_old = p.app_k != nullptr ? n - p.app_add.n[b] : n;  // tokens below are in kv_local / the host cache
    const int n_loc = p.n_sink + p.n_window;
    const __half* local0 = p.att_local + bh * (size_t)n_loc * 2 * TKV_D;
    const int half = lane / 32, l32 = lane % 32;
    float qv[4][4];  // key lanes: this lane's 4 channels of the 4 query heads, times scale2
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint2 w = make_uint2(0u, 0u);
      if (j < G && half == 0) w = reinterpret_cast<const uint2*>(p.q + ((size_t)b * p.hq + (size_t)h * G + j) * TKV_D)[l32];
      const uint32_t wx = w.x, wy = w.y;
      const half2_t a = __builtin_bit_cast(half2_t, wx), c = __builtin_bit_cast(half2_t, wy);
      qv[j][0] = (float)a[0] * p.att_scale2, qv[j][1] = (float)a[1] * p.att_scale2;
      qv[j][2] = (float)c[0] * p.att_scale2, qv[j][3] = (float)c[1] * p.att_scale2;
    }
    float m_run[4], l_run[4], o_run[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      m_run[j] = -INFINITY, l_run[j] = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c) o_run[j][c] = 0.f;
    }
    // the R rows of the pass that starts at attended token i0: lane y < R works out where row
    // i0 + y lives (its K half and its V half), then one load instruction per row
    auto fetch = [&](int i0, uint2 (&r)[R]) {
      const __half* kp = local0;
      const __half* vp = local0 + TKV_D;
      if (i0 >= n_res && i0 + R <= n_att) {  // (uniform) the common pass: selected tokens only, rows of the host cache
        // (kept inside the cache whatever a caller's index list holds: with a given selection the
        // entries are the caller's)
        const int tok = min(max(sel[i0 - n_res + (lane < R ? lane : 0)], 0), p.capacity - 1);
        kp = p.att_host + (bh * p.capacity + (size_t)tok) * 2 * TKV_D;
        vp = kp + TKV_D;
      } else {
        const int i = i0 + lane;
        if (lane < R && i < n_att) {
          int tok;
          bool host = false;
          if (i < n_sk) tok = i;
          else if (i < n_res) tok = w0 + (i - n_sk);
          else tok = min(max(sel[i - n_res], 0), p.capacity - 1), host = true;
          if (host) {
            kp = p.att_host + (bh * p.capacity + (size_t)tok) * 2 * TKV_D;
            vp = kp + TKV_D;
          } else if (tok >= n_old) {
            const size_t row = (((size_t)b * p.app_stride + (tok - n_old)) * p.hkv + h) * TKV_D;
            kp = p.app_k + row;
            vp = p.app_v + row;
          } else {
            kp = local0 + (size_t)(tok < p.n_sink ? tok : p.n_sink + tok % p.n_window) * 2 * TKV_D;
            vp = kp + TKV_D;
          }
        }
      }
#pragma unroll
      for (int y = 0; y < R; ++y) {
        const uint64_t ka = (uint64_t)read_lane((uint32_t)(uintptr_t)kp, y) | ((uint64_t)read_lane((uint32_t)((uintptr_t)kp >> 32), y) << 32);
        const uint64_t va = (uint64_t)read_lane((uint32_t)(uintptr_t)vp, y) | ((uint64_t)read_lane((uint32_t)((uintptr_t)vp >> 32), y) << 32);
        // (named as global memory, which pinned host memory is too: loads through generic pointers
        // cannot be counted one by one, and every wait for a row would wait for all rows in flight)
        const tkv::tkv_u32x2 w = reinterpret_cast<const __attribute__((address_space(1))) tkv::tkv_u32x2*>(half == 0 ? ka : va)[l32];
        r[y] = make_uint2(w.x, w.y);
      }
    };
    // one pass: the wave's R rows that start at attended token i0
    auto pass = [&](int i0, const uint2 (&r)[R]) {
      // partial logits of this lane's 4 channels: v[4 y + j]
      float v[R * 4];
#pragma unroll
      for (int y = 0; y < R; ++y) {
        const uint32_t rx = r[y].x, ry = r[y].y;  // (copied out: a bit cast applied to a vector element reads element 0)
        const half2_t a = __builtin_bit_cast(half2_t, rx), c = __builtin_bit_cast(half2_t, ry);
        const float k0 = (float)a[0], k1 = (float)a[1], k2 = (float)c[0], k3 = (float)c[1];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          v[4 * y + j] = __builtin_fmaf(qv[j][3], k3, __builtin_fmaf(qv[j][2], k2, __builtin_fmaf(qv[j][1], k1, qv[j][0] * k0)));
      }
      // sum over the 32 key lanes: every exchange halves the values a lane is responsible for
      int base = 0;
      auto halve = [&](auto dist, auto count) {  // lanes that differ in bit `dist` split `2 count` values between them
        constexpr int D = decltype(dist)::value, C = decltype(count)::value;
        const bool up = (lane & D) != 0;
        if (C >= 1) {
#pragma unroll
          for (int x = 0; x < (C >= 1 ? C : 1); ++x) {
            const float lo = v[x], hi = v[x + C];
            v[x] = (up ? hi : lo) + swap_xor<D>(up ? lo : hi);
          }
          base += up ? C : 0;
        } else {  // one value left per lane: both partners keep the sum
          v[0] += swap_xor<D>(v[0]);
        }
      };
      using std::integral_constant;
      halve(integral_constant<int, 16>{}, integral_constant<int, R * 2>{});
      halve(integral_constant<int, 8>{}, integral_constant<int, R>{});
      halve(integral_constant<int, 4>{}, integral_constant<int, R / 2>{});
      halve(integral_constant<int, 2>{}, integral_constant<int, R / 4>{});
      halve(integral_constant<int, 1>{}, integral_constant<int, R / 8>{});
      if (half == 0) {  // logits base, base + 1, ... of this key lane
#pragma unroll
        for (int z = 0; z < (R >= 8 ? R / 8 : 1); ++z) xs[base + z] = v[z];
      }
      // (a wave's LDS operations execute in order: the reads below see the writes above)
      // online softmax and weighted V sum; value lanes own 4 channels each
      float xa[R * 4];  // logits [y][j]
#pragma unroll
      for (int z = 0; z < R; ++z) {
        const float4 t = *reinterpret_cast<const float4*>(xs + 4 * z);
        xa[4 * z] = t.x, xa[4 * z + 1] = t.y, xa[4 * z + 2] = t.z, xa[4 * z + 3] = t.w;
      }
      float vf[R][4];  // this lane's 4 channels of the rows (value lanes: of V)
#pragma unroll
      for (int y = 0; y < R; ++y) {
        const uint32_t rx = r[y].x, ry = r[y].y;
        const half2_t a = __builtin_bit_cast(half2_t, rx), c = __builtin_bit_cast(half2_t, ry);
        vf[y][0] = (float)a[0], vf[y][1] = (float)a[1], vf[y][2] = (float)c[0], vf[y][3] = (float)c[1];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float x[R], mx = -INFINITY;
#pragma unroll
        for (int y = 0; y < R; ++y) {
          x[y] = i0 + y < n_att ? xa[4 * y + j] : -INFINITY;
          mx = fmaxf(mx, x[y]);
        }
        if (mx > m_run[j]) {  // (uniform over the wave) a new maximum: the sums so far shrink
          const float alpha = __builtin_amdgcn_exp2f(m_run[j] - mx);
          l_run[j] *= alpha;
#pragma unroll
          for (int c = 0; c < 4; ++c) o_run[j][c] *= alpha;
          m_run[j] = mx;  // finite: the pass holds at least one token
        }
#pragma unroll
        for (int y = 0; y < R; ++y) {
          const float pw = __builtin_amdgcn_exp2f(x[y] - m_run[j]);
          l_run[j] += pw;
#pragma unroll
          for (int c = 0; c < 4; ++c) o_run[j][c] = __builtin_fmaf(pw, vf[y][c], o_run[j][c]);
        }
      }
    };
    // Two passes of rows are in flight while a third is worked on: a wave that has nothing on its
    // way while it computes leaves the host link idle for that long.  Every request is issued
    // whether or not the pass exists (past the end: the head's first resident row, unused), so
    // that the number of loads behind the rows a pass waits for is the same on every path.
    constexpr int kStride = kWavesPerBlock * R;
    uint2 ra[R], rb[R];
    TKV_PH(8);
    fetch(wave * R, ra);
    fetch(wave * R + kStride, rb);
    for (int i0 = wave * R; i0 < n_att; i0 += 2 * kStride) {
      pass(i0, ra);
      fetch(i0 + 2 * kStride, ra);
      if (i0 + kStride < n_att) pass(i0 + kStride, rb);
      fetch(i0 + 3 * kStride, rb);
    }
    TKV_PH(9);
    TKV_PHW(16 + wave);
    // The waves' results meet in the list area, which nothing has used since the selection.
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float* dst = mrg + (wave * 4 + j) * (TKV_D + 4);
      if (lane == 0) *reinterpret_cast<float2*>(dst) = make_float2(m_run[j], l_run[j]);
      if (half == 1) *reinterpret_cast<float4*>(dst + 4 + 4 * l32) = make_float4(o_run[j][0], o_run[j][1], o_run[j][2], o_run[j][3]);
    }
    __syncthreads();
    TKV_PH(10);
    // one thread per query head and four channels: 16-byte reads of the waves' partial sums,
    // every element summed over the waves in ascending order
    if (tid < 4 * (TKV_D / 4) && tid / (TKV_D / 4) < G) {
      const int j = tid / (TKV_D / 4), c4 = tid % (TKV_D / 4);
      float2 ml[kWavesPerBlock];
      float M = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) {
        ml[w] = *reinterpret_cast<const float2*>(mrg + (w * 4 + j) * (TKV_D + 4));
        M = fmaxf(M, ml[w].x);
      }
      float L = 0.f, O[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) {
        const float4 o = *reinterpret_cast<const float4*>(mrg + (w * 4 + j) * (TKV_D + 4) + 4 + 4 * c4);
        const float wgt = ml[w].x == -INFINITY ? 0.f : exp2f(ml[w].x - M);
        L = __builtin_fmaf(ml[w].y, wgt, L);
        O[0] = __builtin_fmaf(o.x, wgt, O[0]), O[1] = __builtin_fmaf(o.y, wgt, O[1]);
        O[2] = __builtin_fmaf(o.z, wgt, O[2]), O[3] = __builtin_fmaf(o.w, wgt, O[3]);
      }
      __half r[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) r[c] = __float2half_rn(L > 0.f ? O[c] / L : 0.f);
      uint2 packed;
      __builtin_memcpy(&packed, r, 8);
      *reinterpret_cast<uint2*>(p.att_out + ((size_t)b * p.hq + (size_t)h * G + j) * TKV_D + 4 * c4) = packed;
    }
    TKV_PH(11);
  };

  // Scoring, listing and, in the head's last workgroup, the selection.  Returns true in the
  // workgroup that holds the head's selected tokens at the end (false everywhere else).
  int given_cnt = 0;
  auto select_tokens = [&]() -> bool {
    if (ATT && p.given != 0) {  // selected by an earlier call: copy the list, then fetch and attend
      if (blockIdx.x != 0) return false;
      given_cnt = max(0, min(p.topk_count[bh], p.top_k));
      for (int i = tid; i < given_cnt; i += kThreads) sel_s[i] = out[i];
      return true;
    }
    if (k == 0 && blockIdx.x == 0) {  // nothing to select: the first workgroup reports the empty result
      for (int i = tid; i < p.top_k; i += kThreads) out[i] = -1;
      if (tid == 0) p.topk_count[bh] = 0;
    }
    const int t0 = blockIdx.x * p.tpw;
    appends = k == 0 && blockIdx.x == 0;  // no candidates, no arrivals
    if (ATT && k == 0) return blockIdx.x == 0;  // ... and attends to what is resident
    if (t0 >= n) return false;
    const int t_end = min(n, t0 + p.tpw);  // this workgroup's tokens: [t0, t_end), kTok per pass
    const int nblk = (n + p.tpw - 1) / p.tpw;
    TKV_PH(0);
    for (int i = tid; i < kBins; i += kThreads) hist[i] = 0u;
    // Stage 1 fused in (resident channel-major keys only): every workgroup derives the head's
    // channel list for itself, the first one also reports it
    __shared__ int32_t s_chan[DS];
    const bool dyn = CM && p.k_absmax != nullptr;
    if (dyn) {
      __shared__ float s_s[TKV_D];
      __shared__ uint32_t s_sel[TKV_D];
      __shared__ __half q_all[GH][TKV_D];  // whole query rows, fetched while the list is being made
      if (tid >= kThreads - GH * TKV_D / 2) {
        const int x = tid - (kThreads - GH * TKV_D / 2), j = x / (TKV_D / 2), w = x % (TKV_D / 2);
        const uint32_t v = j < G ? reinterpret_cast<const uint32_t*>(p.q + ((size_t)b * p.hq + (size_t)h * G + j) * TKV_D)[w] : 0u;
        reinterpret_cast<uint32_t*>(&q_all[j][0])[w] = v;
      }
      tkv::select_channels_block(p.q_hat + ((size_t)b * p.hq + (size_t)h * G) * TKV_D, G, p.k_absmax + bh * TKV_D, DS,
                                 s_s, s_sel, s_chan, blockIdx.x == 0 ? p.channel_out + bh * DS : nullptr);
      if (tid < GH * DS) {
        const int j = tid / DS, i = tid % DS;
        qc[j][i] = __half2float(q_all[j][s_chan[i]]);  // rows of heads >= G are zero
      }
    } else if (tid < GH * DS) {
      const int j = tid / DS, i = tid % DS;
      const int c = p.channel_idx[bh * DS + i];
      qc[j][i] = j < G ? __half2float(p.q[((size_t)b * p.hq + (size_t)h * G + j) * TKV_D + c]) : 0.f;
    }
    // all of a thread's rows of a pass are requested before the first is used (threads past
    // the share's last token re-read that token: no traffic beyond the share)
    static_assert(DS % 4 == 0, "summary rows are read in 8-byte pieces");
    uint2 rows[kPer][DS / 4];  // (pairs of pieces merge into 16-byte loads where the row allows it)
    uint2 cols[DS];  // CM: four consecutive tokens of every channel row
    auto load_pass = [&](int tb, int te, auto n_rows) {
      if (CM) {
        static_assert(kPer == 4, "four tokens per 8-byte load");
        const int tq = min(tb + kPer * tid, (te - 1) & ~3);  // past the end: the share's last group of four
  #pragma unroll
        for (int i = 0; i < DS; ++i) {
          const int row = dyn ? s_chan[i] : p.rows_per_head == DS ? i : p.channel_idx[bh * DS + i];
          cols[i] = *reinterpret_cast<const uint2*>(p.summary + (bh * p.rows_per_head + row) * (size_t)p.capacity + tq);
        }
      } else {
        const __half* srow = p.summary + (bh * p.capacity) * DS;
  #pragma unroll
        for (int it = 0; it < decltype(n_rows)::value; ++it) {
          const int t = min(tb + it * kThreads + tid, te - 1);  // past the end: the share's last row again
          if (DS % 8 == 0) {
  #pragma unroll
            for (int x = 0; x < DS / 8; ++x) {
              const uint4 v = reinterpret_cast<const uint4*>(srow + (size_t)t * DS)[x];
              rows[it][2 * x] = make_uint2(v.x, v.y);
              rows[it][2 * x + 1] = make_uint2(v.z, v.w);
            }
          } else {
  #pragma unroll
            for (int x = 0; x < DS / 4; ++x) rows[it][x] = reinterpret_cast<const uint2*>(srow + (size_t)t * DS)[x];
          }
        }
      }
    };
    if (k == 0) return false;  // (after Stage 1: the channel list is reported even when no token is a candidate)
    load_pass(t0, t_end, std::integral_constant<int, kPer>{});
    __syncthreads();
    // query channels into registers (heads >= G are zero: adding their +0 sums changes nothing)
    // kept as fp16 pairs: the multiply-adds below convert both operands on the fly (exactly)
    uint32_t qr[4][DS / 2];
  #pragma unroll
    for (int j = 0; j < 4; ++j)
  #pragma unroll
      for (int i = 0; i < DS / 2; ++i)
        qr[j][i] = GH == 4 ? __builtin_bit_cast(uint32_t, half2_t{(_Float16)qc[j][2 * i], (_Float16)qc[j][2 * i + 1]}) : 0u;

    // Keys of the loaded pass `ps` of the share [ts, te): kb[kPer * ps + j] is the key of token
    // ts + ps * kTok + j * kThreads + tid (0 for a non-candidate or past the share).  Token-major
    // keys are produced in that order; channel-major ones (token ts + ps * kTok + 4 tid + it) go
    // through `stage` and are put in order by collect_keys.
    uint32_t kb[kSub];
    // (q_from_lds: the re-scoring of another share in the slow path reads the query channels from
    // LDS instead of keeping 64 registers alive through the common path)
    auto score_pass = [&](int ts, int te, int ps, bool count, auto q_from_lds, auto n_rows) {
      const int tb = ts + ps * kTok;
      int tid_again = tid;  // opaque copy: the token numbers are worked out again here rather than
      asm volatile("" : "+v"(tid_again));  // kept in registers (or spilled) since the loads were issued
  #pragma unroll
      for (int it = 0; it < (CM ? kPer : decltype(n_rows)::value); ++it) {
        const int t = CM ? tb + kPer * tid_again + it : tb + it * kThreads + tid_again;
        _Float16 kx[DS];
        if (CM) {
  #pragma unroll
          for (int i = 0; i < DS; ++i) {
            const uint32_t wy = it < 2 ? cols[i].x : cols[i].y;
            const half2_t hh = __builtin_bit_cast(half2_t, wy);
            kx[i] = hh[it % 2];
          }
        } else {
  #pragma unroll
          for (int x = 0; x < DS / 4; ++x) {
            const uint32_t w[2] = {rows[it][x].x, rows[it][x].y};
  #pragma unroll
            for (int y = 0; y < 2; ++y) {
              const uint32_t wy = w[y];
              const half2_t hh = __builtin_bit_cast(half2_t, wy);
              kx[4 * x + 2 * y] = hh[0];
              kx[4 * x + 2 * y + 1] = hh[1];
            }
          }
        }
        float total = 0.f;
        // (groups of 5 to 8: the query channels are read from LDS again for every token rather than
        // held in 128 registers across the pass)
        if (GH > 4) asm volatile("" ::: "memory");
  #pragma unroll
        for (int j = 0; j < GH; ++j) {
          // left-to-right sum of exact products: fma(q, k, a) rounds once, like a + q*k; the
          // first term fma(q, k, +0) is the exact product (only the sign of a zero can differ,
          // and the final + 0.0f removes that)
          constexpr bool kLdsQ = GH > 4 || decltype(q_from_lds)::value;
          float a = 0.f;
  #pragma unroll
          for (int i = 0; i < DS; i += 2) {
            float q0, q1;
            if (kLdsQ) {
              q0 = qc[j][i], q1 = qc[j][i + 1];
            } else {
              // (opaque copy: keeps the pair packed in one register instead of two converted ones
              // held across the whole pass)
              uint32_t w = qr[j % 4][i / 2];
              asm volatile("" : "+v"(w));
              const half2_t hq = __builtin_bit_cast(half2_t, w);
              q0 = (float)hq[0], q1 = (float)hq[1];
            }
            a = __builtin_fmaf(q0, (float)kx[i], a);
            a = __builtin_fmaf(q1, (float)kx[i + 1], a);
          }
          total = j == 0 ? a : total + a;
        }
        total = total + 0.0f;
        uint32_t key = 0u;  // non-candidates: below every score
        if (t < te && t >= lo && t < hi) {
          key = score_key(total);
          if (count) atomicAdd(&hist[key >> kLowBits], 1u);
        }
        if (CM)
          stage[ps * kTok + kPer * tid + it] = key;
        else
          kb[kPer * ps + it] = key;
      }
    };
    // scores the whole share [ts, te) (the first pass already loaded if `loaded`)
    // the first kTok tokens in one pass, the rest (at most one sub-tile) in a second, short one
    auto score_share = [&](int ts, int te, bool loaded, bool count, auto q_from_lds) {
      using Full = std::integral_constant<int, kPer>;
      using One = std::integral_constant<int, 1>;
      if (!loaded) load_pass(ts, te, Full{});
      score_pass(ts, te, 0, count, q_from_lds, Full{});
      if (ts + kTok < te) {
        load_pass(ts + kTok, te, One{});
        score_pass(ts, te, 1, count, q_from_lds, One{});
      } else if (!CM) {
        kb[kPer] = 0u;
      }
      if (CM) {
        __syncthreads();
  #pragma unroll
        for (int j = 0; j < kSub; ++j) kb[j] = ts + j * kThreads + tid < te ? stage[j * kThreads + tid] : 0u;
      }
    };
    // Lists the keys kb of the share starting at token ts that lie in or above `bin`, in token
    // order, from entry ts of the head's list area; returns the list length (in every thread).
    uint2* list_g = p.ws.cand + bh * p.ws.cand_stride;  // the workgroup of share x owns entries [x * tpw, +tpw)
    auto list_share = [&](int ts, uint32_t bin, bool first_use) -> uint32_t {
      unsigned long long mask[kSub];
  #pragma unroll
      for (int j = 0; j < kSub; ++j) mask[j] = __builtin_amdgcn_ballot_w64(kb[j] != 0u && (kb[j] >> kLowBits) >= bin);
      uint32_t before[kSub];
      if (!first_use) __syncthreads();  // s_cnt may still be read by the previous use
      const uint32_t total = subtile_offsets(mask, &s_cnt[0][0], wave, lane, before);
  #pragma unroll
      for (int j = 0; j < kSub; ++j) {
        if ((mask[j] >> lane) & 1ull) {
          uint2* e = &list_g[(size_t)ts + before[j] + rank_in(mask[j])];
          st_agent(&e->x, kb[j]);
          st_agent(&e->y, (uint32_t)(ts + j * kThreads + tid));
        }
      }
      return total;
    };

    score_share(t0, t_end, true, true, std::false_type{});
    __syncthreads();
    TKV_PH(1);
    // ---- `my_bin`: the bin of this workgroup's r-th key, down to which it lists its tokens
    uint32_t* ctrl = p.ws.ctrl + bh * kCtrlWords;
    uint32_t* cnt_g = p.ws.blk + bh * p.ws.nblk_cap;
    constexpr int kOwn = kBins / kThreads;  // bins per thread, descending: kBins - 1 - (kOwn * tid + i)
    static_assert(kOwn == 8, "two 16-byte reads per thread");
    {
      const uint32_t mine = (uint32_t)max(0, min(hi, t_end) - max(lo, t0));  // candidates in this share
      // fair share of k, times 1.5, plus 16
      const uint32_t r = (uint32_t)(((unsigned long long)k * mine * 3ull) / (2ull * (unsigned long long)(hi - lo))) + 16u;
      const uint32_t ranks[1] = {r < mine ? r : 0u};  // (fewer candidates than that: all of them are listed)
      uint32_t c[kOwn];
      {
        const uint4 w0 = *reinterpret_cast<const uint4*>(&hist[kBins - kOwn * tid - kOwn]);
        const uint4 w1 = *reinterpret_cast<const uint4*>(&hist[kBins - kOwn * tid - kOwn + 4]);
        c[7] = w0.x, c[6] = w0.y, c[5] = w0.z, c[4] = w0.w, c[3] = w1.x, c[2] = w1.y, c[1] = w1.z, c[0] = w1.w;
      }
      find_ranks<1, kOwn>(c, ranks, s_wtot, s_res, wave, lane);
      const uint32_t my_bin = s_res[0];
      const uint32_t my_len = list_share(t0, my_bin, true);
      if (tid == 0) st_agent(&cnt_g[blockIdx.x], (my_bin << kCountBits) | my_len);
    }
    TKV_PH(2);
    // (what the head's last workgroup needs cleared is cleared by every workgroup here, under the
    // wait for the list stores: one barrier less on the path that everything after waits for)
    __shared__ uint32_t r1[2048], r2[2048], r3[1024];  // radix-select histograms: 11 + 11 + 10 key bits
    __shared__ uint32_t lens[kThreads], lbin[kThreads];  // list length and bin L of every share
    __shared__ uint32_t s_lmax, s_lmin, s_nsame;
    for (int i = tid; i < 2048; i += kThreads) r1[i] = 0u, r2[i] = 0u;
    r3[tid] = 0u;
    if (tid == 0) s_lmax = 0u, s_lmin = kBins - 1, s_nsame = 0u;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      const uint32_t before = atomicAdd(&ctrl[kDone2], 1u);
      scratch[kWavesPerBlock + 2] = before == (uint32_t)nblk - 1u;
      scratch[kWavesPerBlock + 3] = before == 0u;
    }
    __syncthreads();
    appends = scratch[kWavesPerBlock + 3] != 0u;
    TKV_PH(3);
    if (!scratch[kWavesPerBlock + 2]) {
      if (ATT && p.pf != nullptr) {
        // This workgroup's own share of that summary (the workgroup with the same number will
        // score it in the next launch): HBM is idle from here on, and the next launch then finds
        // the rows in the memory-side cache.  Eight 16-byte loads per thread in flight; the
        // values are only combined so that the loads are not dropped.
        // (not at once: the head's last workgroup is about to read the lists through the same
        // memory system, and the selection waits for that round trip)
        __builtin_amdgcn_s_sleep(127);
        __builtin_amdgcn_s_sleep(127);
        const uint4* src = reinterpret_cast<const uint4*>(p.pf + (bh * p.capacity + (size_t)t0) * DS);
        const int n_vec = max(0, t_end - t0) * DS / 8;
        uint32_t mix = 0;
        for (int i = tid; i < n_vec; i += 8 * kThreads) {
          uint4 w[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) w[j] = src[min(i + j * kThreads, n_vec - 1)];
#pragma unroll
          for (int j = 0; j < 8; ++j) mix ^= w[j].x ^ w[j].y ^ w[j].z ^ w[j].w;
        }
        asm volatile("" ::"v"(mix));
      }
      return false;
    }

    // ---- the head's last workgroup.  One round of device-scope loads brings the workgroups'
    // control words and the first `spec` entries of every list (entry e = i * kThreads + tid of
    // the round belongs to share e / spec, so ascending e is token order); spec is a power of two
    // a quarter above the nominal list length, the round never fetches more than kSub entries per thread.
    int spec_shift = 0;
    {
      const uint32_t nominal = (3u * k) / (2u * (uint32_t)nblk) + 16u;
      while ((1u << spec_shift) < nominal + nominal / 4u) ++spec_shift;
      while (spec_shift > 0 && ((size_t)nblk << spec_shift) > (size_t)kSub * kThreads) --spec_shift;
    }
    uint32_t ek[kSub], et[kSub];  // this thread's entries: key and token
    bool fits;
    {
      const tkv::AgentBuf cb(cnt_g, (uint32_t)nblk * 4u), lb(list_g, (uint32_t)min((size_t)n * 8, (size_t)0xFFFFFFF0u));
      const uint32_t cw = cb.x1((uint32_t)tid * 4u);  // 0 beyond the head's workgroups (fewer than 1024)
  #pragma unroll
      for (int i = 0; i < kSub; ++i) {
        const uint32_t e = (uint32_t)(i * kThreads + tid), x = e >> spec_shift, off = e & ((1u << spec_shift) - 1u);
        const bool want = x < (uint32_t)nblk && off < (uint32_t)p.tpw;
        const tkv::tkv_u32x2 v = lb.x2(want ? (x * (uint32_t)p.tpw + off) * 8u : tkv::AgentBuf::kNone);
        ek[i] = v.x;
        et[i] = v.y;
      }
      if (tid == 0) st_agent(&ctrl[kDone2], 0u);  // left zero for the next call
      for (int i = (int)k + tid; i < p.top_k; i += kThreads) out[i] = -1;
      if (tid == 0) p.topk_count[bh] = (int32_t)k;
      const uint32_t len = cw & ((1u << kCountBits) - 1u);
      lens[tid] = len;
      lbin[tid] = cw >> kCountBits;
      // largest L of the head: one atomic per wave
      uint32_t lm = cw >> kCountBits;
  #pragma unroll
      for (int m = 32; m >= 1; m >>= 1) lm = max(lm, (uint32_t)__shfl_xor((int)lm, m, 64));
      if (lane == 0 && lm != 0u) atomicMax(&s_lmax, lm);
      // lowest L among the shares that list anything (every listed key lies in or above it)
      uint32_t ln = tid < nblk && len != 0u ? cw >> kCountBits : (uint32_t)kBins - 1u;
  #pragma unroll
      for (int m = 32; m >= 1; m >>= 1) ln = min(ln, (uint32_t)__shfl_xor((int)ln, m, 64));
      if (lane == 0) atomicMin(&s_lmin, ln);
      fits = __syncthreads_or(len > (1u << spec_shift) ? 1 : 0) == 0;
    }
    TKV_PH(4);

    // k-th largest key of a set of keys (each thread offers its own through `each`), by radix
    // select over three digits of 11, 11 and s1 - 11 bits, the first being (key >> s1) - base,
    // clamped to 2047; every search is done by the whole workgroup (two or one bin per thread).
    // s1 = 21, base = 0 covers all 32 bits of any key.  The listed keys share their leading bits,
    // though, and LDS atomics of a wave on one address are executed one after the other: with
    // s1 = kFastShift and base = (lowest bin L of any list) << (kLowBits - kFastShift) the first
    // digits spread over hundreds of values and few keys share the k-th key's digit, at the price
    // of keys more than four binades above that bin being clamped: returns false if the k-th
    // key is among those (the caller then falls back to s1 = 21).
    // T: the key; take: how many keys equal to T belong to the k largest.  The three histograms
    // and s_nsame must be zero.
    auto kth_key = [&](auto each, int s1, uint32_t base, uint32_t& T, uint32_t& take) -> bool {
      uint32_t k_rem = k;
      auto search2 = [&](const uint32_t* hist, uint32_t& digit) {  // 2048 bins
        const uint2 w = *reinterpret_cast<const uint2*>(&hist[2048 - 2 * tid - 2]);
        const uint32_t c[2] = {w.y, w.x};
        const uint32_t ranks[1] = {k_rem};
        find_ranks<1, 2>(c, ranks, s_wtot, s_res, wave, lane);
        digit = s_res[0];
        k_rem -= s_res[1];
      };
      const int s2 = s1 - 11;
      const uint32_t low_mask = (1u << s2) - 1u;
      uint32_t d1, d2, d3;
      each([&](uint32_t key) { if (key != 0u) atomicAdd(&r1[min((key >> s1) - base, 2047u)], 1u); });
      __syncthreads();
      TKV_PH(6);
      search2(r1, d1);
      if (s1 != 21 && d1 == 2047u) return false;
      const uint32_t top = d1 + base;
      // Keys that share the first digit: usually a few dozen.  Up to 1024 of them are collected
      // in LDS (in any order) and ranked against each other directly; more go through two more
      // digits.
      const uint32_t n_same = r1[d1];
      if (n_same <= (uint32_t)kThreads) {
        // (s_nsame is zero: cleared with the histograms)
        each([&](uint32_t key) { if (key != 0u && (key >> s1) == top) r2[atomicAdd(&s_nsame, 1u)] = key; });
        __syncthreads();
        // the k_rem-th largest of them: the key v with fewer than k_rem keys above it and at least
        // k_rem keys at or above it (every thread that holds such a key reports the same result)
        if ((uint32_t)tid < n_same) {
          const uint32_t v = r2[tid];
          uint32_t gt = 0, ge = 0;
          for (uint32_t y = 0; y < n_same; ++y) {
            const uint32_t o = r2[y];
            gt += o > v ? 1u : 0u;
            ge += o >= v ? 1u : 0u;
          }
          if (gt < k_rem && k_rem <= ge) s_res[0] = v, s_res[1] = k_rem - gt;
        }
        __syncthreads();
        T = s_res[0];
        take = s_res[1];
        return true;
      }
      each([&](uint32_t key) { if ((key >> s1) == top) atomicAdd(&r2[(key >> s2) & 0x7FFu], 1u); });
      __syncthreads();
      search2(r2, d2);
      const uint32_t top2 = (top << 11) | d2;
      each([&](uint32_t key) { if ((key >> s2) == top2) atomicAdd(&r3[key & low_mask], 1u); });
      __syncthreads();
      {
        const uint32_t c[1] = {r3[1023 - tid]};
        const uint32_t ranks[1] = {k_rem};
        find_ranks<1, 1>(c, ranks, s_wtot, s_res, wave, lane);
        d3 = s_res[0];
        take = k_rem - s_res[1];
      }
      T = (top2 << s2) | d3;
      return true;
    };

    if (fits) {
      // ---- every list entry is in a register of some thread
  #pragma unroll
      for (int i = 0; i < kSub; ++i) {
        const uint32_t e = (uint32_t)(i * kThreads + tid), x = e >> spec_shift, off = e & ((1u << spec_shift) - 1u);
        if (!(x < (uint32_t)nblk && off < lens[x])) ek[i] = 0u;  // beyond the list: below every key
      }
      uint32_t T, take;
      const bool found = kth_key([&](auto f) {
  #pragma unroll
        for (int i = 0; i < kSub; ++i) f(ek[i]);
      }, kFastShift, s_lmin << (kLowBits - kFastShift), T, take);
      TKV_PH(5);
      // Every list is complete down to its bin L, so T is the head's exact k-th key if no L lies
      // above T's bin (a token missing from a list is then below T).
      if (found && (T >> kLowBits) >= s_lmax) {
        // ordered compaction: every key above T, and the first `take` equal to T
        unsigned long long mg[kSub], me[kSub];
  #pragma unroll
        for (int i = 0; i < kSub; ++i) {
          mg[i] = __builtin_amdgcn_ballot_w64(ek[i] > T);
          me[i] = __builtin_amdgcn_ballot_w64(ek[i] == T);
        }
        uint32_t bg[kSub], be[kSub];
        subtile_offsets2(mg, me, &s_cnt[0][0], &s_cnt2[0][0], wave, lane, bg, be);
  #pragma unroll
        for (int i = 0; i < kSub; ++i) {
          const uint32_t my_gt = bg[i] + rank_in(mg[i]), my_eq = be[i] + rank_in(me[i]);
          int pos = -1;
          if (ek[i] > T) pos = (int)(my_gt + min(my_eq, take));
          else if (ek[i] == T && my_eq < take) pos = (int)(my_gt + my_eq);
          if (pos >= 0) {
            out[pos] = (int32_t)et[i];
            if (ATT) sel_s[pos] = (int32_t)et[i];
          }
        }
        TKV_PH(7);
        return true;
      }
    }

    // ---- slow path: lists longer than the round fetched, or lists that stop above the bin of the
    // k-th key.  Round 0 works on the lists as they are; if its k-th key lies in a bin below some
    // list's L, those shares are re-scored here and listed down to that bin, and round 1 is exact:
    // more entries can only raise the k-th key, and every list is now complete down to a bin at or
    // below it.
    uint32_t T = 0, take = 0, M = 0;
    auto get = [&](uint32_t i) -> uint2 {
      if (i < (uint32_t)kListCap) return list_s[i];
      int x0 = 0, x1 = nblk;  // workgroup whose list holds entry i: offs[x0] <= i < offs[x0 + 1]
      while (x1 - x0 > 1) {
        const int mid = (x0 + x1) / 2;
        if (offs[mid] <= i) x0 = mid; else x1 = mid;
      }
      const uint2* e = &list_g[(size_t)x0 * p.tpw + (i - offs[x0])];
      return make_uint2(ld_agent(&e->x), ld_agent(&e->y));
    };
    for (int round = 0; round < 2; ++round) {
      // concatenate the lists (wave w copies those of workgroups w, w + 16, ...): entry i of the
      // concatenation lives in LDS if i < kListCap, else it is read from its list in the workspace
      __syncthreads();
      for (int i = tid; i < 2048; i += kThreads) r1[i] = 0u, r2[i] = 0u;
      r3[tid] = 0u;
      if (tid == 0) s_nsame = 0u;
      if (tid < 64) {  // exclusive scan of the list lengths by one wave
        uint32_t carry = 0;
        for (int x0 = 0; x0 < nblk; x0 += 64) {
          const int x = x0 + tid;
          const uint32_t c = x < nblk ? lens[x] : 0u;
          const uint32_t incl = wave_prefix_incl(c);
          if (x < nblk) offs[x] = carry + incl - c;
          carry += read_lane(incl, 63);
        }
        if (tid == 0) offs[nblk] = carry;
      }
      __syncthreads();
      M = offs[nblk];
      for (int x = wave; x < nblk; x += kWavesPerBlock) {
        const uint32_t o = offs[x], c = offs[x + 1] - o;
        for (uint32_t i = lane; i < c; i += 64) {
          if (o + i < (uint32_t)kListCap) {
            const uint2* e = &list_g[(size_t)x * p.tpw + i];
            list_s[o + i] = make_uint2(ld_agent(&e->x), ld_agent(&e->y));
          }
        }
      }
      __syncthreads();
      kth_key([&](auto f) {
        for (uint32_t i = tid; i < M; i += kThreads) f(get(i).x);
      }, 21, 0u, T, take);
      if (round == 1) break;
      const uint32_t tbin = T >> kLowBits;
      if (tid == 0) s_nrep = 0u;
      __syncthreads();
      if (tid < nblk && lbin[tid] > tbin) s_rep[atomicAdd(&s_nrep, 1u)] = (uint16_t)tid;
      __syncthreads();
      const uint32_t nrep = s_nrep;
      if (nrep == 0u) break;
      for (uint32_t r = 0; r < nrep; ++r) {
        const int x = s_rep[r];
        const int ts = x * p.tpw, te = min(n, ts + p.tpw);
        score_share(ts, te, false, false, std::true_type{});
        const uint32_t relen = list_share(ts, tbin, false);
        if (tid == 0) lens[x] = relen, lbin[x] = tbin;
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the rebuilt lists are read back in round 1
    }
    TKV_PH(6);

    // ordered compaction of the list: every key above T, and the first `take` equal to T
    uint32_t gt_run = 0, eq_run = 0;
    for (uint32_t base = 0; base < M; base += kThreads) {
      const uint32_t i = base + tid;
      uint2 e = make_uint2(0u, 0u);
      if (i < M) e = get(i);
      const bool gt = e.x > T, eq = e.x == T;  // T != 0: every real key has a non-zero prefix
      const unsigned long long mg = __builtin_amdgcn_ballot_w64(gt), me = __builtin_amdgcn_ballot_w64(eq);
      const int set = (int)((base / kThreads) & 1u) * 2;  // alternate the count rows: one barrier per tile
      if (lane == 0) {
        s_cnt[set][wave] = (uint32_t)__builtin_popcountll(mg);
        s_cnt[set + 1][wave] = (uint32_t)__builtin_popcountll(me);
      }
      __syncthreads();
      uint32_t pg = 0, pe = 0, tg = 0, te = 0;
      for (int w = 0; w < kWavesPerBlock; ++w) {
        const uint32_t cg = s_cnt[set][w], ce = s_cnt[set + 1][w];
        pg += w < wave ? cg : 0u;
        pe += w < wave ? ce : 0u;
        tg += cg;
        te += ce;
      }
      const uint32_t my_gt = gt_run + pg + rank_in(mg), my_eq = eq_run + pe + rank_in(me);
      int pos = -1;
      if (gt) pos = (int)(my_gt + min(my_eq, take));
      else if (eq && my_eq < take) pos = (int)(my_gt + my_eq);
      if (pos >= 0) {
        out[pos] = (int32_t)e.y;
        if (ATT) sel_s[pos] = (int32_t)e.y;
      }
      gt_run += tg;
      eq_run += te;
    }
    TKV_PH(7);
    return true;
  };
  const bool holds_selection = select_tokens();
  if (ATT && holds_selection) {
    __syncthreads();  // the selected tokens are in LDS, the scratch areas of the selection are free
    attend(sel_s, p.given != 0 ? given_cnt : (int)k);
  }
  if (p.app_k != nullptr && appends) append_tokens<DS>(p, b, h, tid);  // Eq. 2
}

}  // namespace

#ifdef TKV_PHASE
static void* g_topk_prof = nullptr;
extern "C" void tkv_debug_set_dump_topk(void* ptr) { g_topk_prof = ptr; }
#endif

namespace {
template <int DS, bool CM, bool ATT, int GH = 4>
int32_t launch_fused(const TopkParams& p, dim3 grid, hipStream_t s) {
  // more than 64 KiB of dynamic LDS needs an opt-in, once per kernel
  static const bool lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_select_kernel<DS, CM, ATT, GH>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLds) == hipSuccess;
  if (!lds_ok) return TKV_E_HIP;
  TKV_LAUNCH((score_select_kernel<DS, CM, ATT, GH>), grid, kThreads, kFusedLds, s, p);
  return TKV_OK;
}

// All entry points: validation, parameters, the launch.  keys: token-major key summary
// (rows_per_head == 0) or channel-major rows.
int32_t estimate_topk_launch(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const void* q, const void* keys,
                             int32_t rows_per_head, const int32_t* channel_idx, int32_t* topk_idx,
                             int32_t* topk_count, void* workspace, size_t workspace_bytes, void* stream,
                             const float* k_absmax = nullptr, const void* q_hat = nullptr,
                             int32_t* channel_out = nullptr, const TopkParams* app = nullptr,
                             const TopkParams* att = nullptr) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !keys || !q || !topk_idx || !topk_count || !workspace) return TKV_E_INVAL;
  if (k_absmax ? (!q_hat || !channel_out) : !channel_idx) return TKV_E_INVAL;
  if ((uintptr_t)keys % 8 != 0) return TKV_E_INVAL;
  const bool cm = rows_per_head != 0;
  if (cm && rows_per_head != d->n_channels && rows_per_head != TKV_D) return TKV_E_INVAL;
  if (cm && d->capacity % 8 != 0) return TKV_E_INVAL;
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
  p.summary = (const __half*)keys;
  p.rows_per_head = rows_per_head;
  p.channel_idx = channel_idx;
  p.k_absmax = k_absmax;
  p.q_hat = (const __half*)q_hat;
  p.channel_out = channel_out;
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
  p.given = 0;
#ifdef TKV_PHASE
  p.prof = (long long*)g_topk_prof;
#endif

  hipStream_t s = (hipStream_t)stream;
  // Tokens per workgroup.  The kernels keep one 1024-thread workgroup per compute unit, so
  // the launch takes ceil(workgroups / compute units) rounds: with 4096 tokens each, a
  // context just past a multiple of 4096 * (compute units / heads) would pay a whole extra
  // round for a few tokens.  Instead the heads' tokens are split evenly over as many
  // workgroups as fill the machine a whole number of times (each owning up to 4096 tokens),
  // or, when even one round is not filled, over more and smaller workgroups.  "The machine" is
  // what the stream may use of it.
  const int n_cus = tkv::stream_compute_units(s);  // of the stream's compute-unit mask, if it has one
  const int bh_count = d->batch * d->n_kv_heads;
  const int full = (max_n + kTok - 1) / kTok;
  int nblk = full > 0 ? full : 1;
  const int per_head = n_cus / bh_count;  // workgroups per head that fill the machine once
  if (per_head >= 1) {
    if (full * bh_count <= n_cus) {
      nblk = (max_n + kThreads - 1) / kThreads;  // at least one token per thread
      if (nblk > per_head) nblk = per_head;
      if (nblk < 1) nblk = 1;
    } else {
      nblk = (full * bh_count / n_cus) * per_head;  // whole rounds, rounded down
    }
  }
  // (a multiple of 16: every workgroup's list starts on a 128-byte line of its own)
  int tpw = ((max_n + nblk - 1) / nblk + 15) & ~15;
  if (tpw < 16) tpw = 16;
  if (tpw > kMaxTpw) {
    tpw = kMaxTpw;
  }
  nblk = (max_n + tpw - 1) / tpw;
  if (nblk < 1) nblk = 1;
  p.tpw = tpw;
  p.app_k = nullptr;
  if (app != nullptr) {
    p.app_k = app->app_k;
    p.app_v = app->app_v;
    p.app_host = app->app_host;
    p.app_local = app->app_local;
    p.app_summary = app->app_summary;
    p.app_stride = app->app_stride;
    p.app_add = app->app_add;
  }
  const dim3 grid(nblk, d->n_kv_heads, d->batch);
  if (nblk >= 1024) return TKV_E_UNSUPPORTED;  // 4 Mi tokens per sequence
  const bool big_group = d->n_q_heads / d->n_kv_heads > 4;  // 5 to 8 query heads per KV head
  if (att != nullptr) {  // token-major summary only
    if (big_group) return TKV_E_UNSUPPORTED;  // (the attention phase holds four heads per lane)
    p.att_host = att->att_host;
    p.att_local = att->att_local;
    p.att_out = att->att_out;
    p.att_scale2 = att->att_scale2;
    p.pf = att->pf;
    if (d->n_channels == 16) return launch_fused<16, false, true>(p, grid, s);
    if (d->n_channels == 12) return launch_fused<12, false, true>(p, grid, s);
    return launch_fused<8, false, true>(p, grid, s);
  }
  if (big_group) {
    if (d->n_channels == 16)
      return cm ? launch_fused<16, true, false, 8>(p, grid, s) : launch_fused<16, false, false, 8>(p, grid, s);
    if (d->n_channels == 12)
      return cm ? launch_fused<12, true, false, 8>(p, grid, s) : launch_fused<12, false, false, 8>(p, grid, s);
    return cm ? launch_fused<8, true, false, 8>(p, grid, s) : launch_fused<8, false, false, 8>(p, grid, s);
  }
  if (d->n_channels == 16)
    return cm ? launch_fused<16, true, false>(p, grid, s) : launch_fused<16, false, false>(p, grid, s);
  if (d->n_channels == 12)
    return cm ? launch_fused<12, true, false>(p, grid, s) : launch_fused<12, false, false>(p, grid, s);
  return cm ? launch_fused<8, true, false>(p, grid, s) : launch_fused<8, false, false>(p, grid, s);
}
}  // namespace

namespace tkv {
// Fetch of the rows of a selection made earlier (topk_idx / topk_count of the same descriptor)
// from the pinned host cache and exact attention, by the attention phase of the one-launch step:
// one workgroup per (sequence, KV head).  Groups of up to 4 query heads, top_k <= 8192 (the list
// is staged in LDS); TKV_E_UNSUPPORTED otherwise, nothing launched.
int32_t launch_fetch_attn(const tkv_sparse_desc* d, const TkvSeqLens& lens, const __half* q, const int32_t* topk_idx,
                          const int32_t* topk_count, const __half* host_rows, const __half* local_rows, __half* out,
                          float scale2, hipStream_t s) {
  if (d->n_q_heads / d->n_kv_heads > 4 || d->top_k > kBins) return TKV_E_UNSUPPORTED;
  TopkParams p = {};
  p.q = q;
  p.topk_idx = const_cast<int32_t*>(topk_idx);
  p.topk_count = const_cast<int32_t*>(topk_count);
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.top_k = d->top_k;
  p.n_sink = d->n_sink;
  p.n_window = d->n_window;
  p.capacity = d->capacity;
  p.tpw = kMaxTpw;
  p.lens = lens;
  p.att_host = host_rows;
  p.att_local = local_rows;
  p.att_out = out;
  p.att_scale2 = scale2;
  p.given = 1;
  return launch_fused<16, false, true>(p, dim3(1, d->n_kv_heads, d->batch), s);
}
}  // namespace tkv

extern "C" int32_t tkv_sparse_estimate_topk(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const void* q,
                                            int32_t* topk_idx, int32_t* topk_count, void* workspace,
                                            size_t workspace_bytes, void* stream) {
  if (!c) return tkv::check_sparse_desc(d) != TKV_OK ? tkv::check_sparse_desc(d) : TKV_E_INVAL;
  return estimate_topk_launch(d, c, q, c->key_summary, 0, c->channel_idx, topk_idx, topk_count, workspace,
                              workspace_bytes, stream);
}

extern "C" int32_t tkv_sparse_estimate_topk_cm(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const void* q,
                                               const int32_t* channel_idx, const void* keys_cm,
                                               int32_t rows_per_head, int32_t* topk_idx, int32_t* topk_count,
                                               void* workspace, size_t workspace_bytes, void* stream) {
  if (rows_per_head == 0) return tkv::check_sparse_desc(d) != TKV_OK ? tkv::check_sparse_desc(d) : TKV_E_INVAL;
  return estimate_topk_launch(d, c, q, keys_cm, rows_per_head, channel_idx, topk_idx, topk_count, workspace,
                              workspace_bytes, stream);
}

extern "C" int32_t tkv_sparse_select_estimate_topk(const tkv_sparse_desc* d, const tkv_sparse_cache* c,
                                                   const tkv_sparse_stage1* s1, const void* q_hat, const void* q,
                                                   int32_t* channel_idx_out, int32_t* topk_idx, int32_t* topk_count,
                                                   void* workspace, size_t workspace_bytes, void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!s1 || !s1->k_absmax || !s1->keys_cm || !q_hat || !channel_idx_out) return TKV_E_INVAL;
  const void* cm = nullptr;  // scored in place: the keys must be resident
  st = tkv::device_view(s1->keys_cm, tkv::kDevDeviceOnly, &cm);
  if (st != TKV_OK) return st;
  return estimate_topk_launch(d, c, q, s1->keys_cm, TKV_D, nullptr, topk_idx, topk_count, workspace, workspace_bytes,
                              stream, s1->k_absmax, q_hat, channel_idx_out);
}

extern "C" int32_t tkv_sparse_append_estimate_topk(const tkv_sparse_desc* d, tkv_sparse_cache* c, const void* k_new,
                                                   const void* v_new, int32_t n_new, const int32_t* n_valid_host,
                                                   const void* q, int32_t* topk_idx, int32_t* topk_count,
                                                   void* workspace, size_t workspace_bytes, void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !c->key_summary || !c->channel_idx || !c->kv_host || !c->kv_local || !k_new || !v_new)
    return TKV_E_INVAL;
  if (n_new < 1 || n_new > 8 || n_new > d->n_window) return TKV_E_INVAL;
  TopkParams app;
  for (int b = 0; b < d->batch; ++b) {
    const int64_t n0 = c->seq_len_host[b];
    const int32_t add = n_valid_host ? n_valid_host[b] : n_new;
    if (n0 < 0 || add < 0 || add > n_new) return TKV_E_INVAL;
    if (n0 + add > d->capacity) return TKV_E_CAPACITY;
    app.app_add.n[b] = add;
  }
  const void* host_dev = nullptr;
  st = tkv::device_view(c->kv_host, tkv::kDevHostOnly, &host_dev);
  if (st != TKV_OK) return st;
  app.app_k = (const __half*)k_new;
  app.app_v = (const __half*)v_new;
  app.app_host = (__half*)host_dev;
  app.app_local = (__half*)c->kv_local;
  app.app_summary = (__half*)c->key_summary;
  app.app_stride = n_new;
  // the kernels see the lengths after the append
  for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] += app.app_add.n[b];
  st = estimate_topk_launch(d, c, q, c->key_summary, 0, c->channel_idx, topk_idx, topk_count, workspace,
                            workspace_bytes, stream, nullptr, nullptr, nullptr, &app);
  if (st != TKV_OK)
    for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] -= app.app_add.n[b];
  return st;
}

extern "C" int32_t tkv_sparse_decode(const tkv_sparse_desc* d, tkv_sparse_cache* c, const void* k_new,
                                     const void* v_new, int32_t n_new, const int32_t* n_valid_host, const void* q,
                                     int32_t* topk_idx, int32_t* topk_count, void* out, float sm_scale,
                                     const void* next_key_summary, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !c->key_summary || !c->channel_idx || !c->kv_host || !c->kv_local || !out)
    return TKV_E_INVAL;
  if ((uintptr_t)next_key_summary % 16 != 0) return TKV_E_INVAL;
  if (n_new < 0 || n_new > 8 || n_new > d->n_window) return TKV_E_INVAL;
  if (n_new > 0 && (!k_new || !v_new)) return TKV_E_INVAL;
  if (d->n_q_heads / d->n_kv_heads > 4) {
    // Groups of 5 to 8 query heads: the attention phase of the one-launch kernel holds four heads
    // per lane.  Two launches instead: append + scoring + Top-K, then fetch + attention (the
    // selection's outputs are the second launch's inputs; `staging` is not used on one stream).
    if (!q || !topk_idx || !topk_count || !workspace) return TKV_E_INVAL;
    st = n_new > 0 ? tkv_sparse_append_estimate_topk(d, c, k_new, v_new, n_new, n_valid_host, q, topk_idx, topk_count,
                                                     workspace, workspace_bytes, stream)
                   : tkv_sparse_estimate_topk(d, c, q, topk_idx, topk_count, workspace, workspace_bytes, stream);
    if (st != TKV_OK) return st;
    return tkv_sparse_gather_attn(d, c, q, topk_idx, topk_count, out, sm_scale, /*staging=*/workspace, workspace,
                                  workspace_bytes, stream, stream);
  }
  TopkParams app, att;
  for (int b = 0; b < d->batch; ++b) {
    const int64_t n0 = c->seq_len_host[b];
    const int32_t add = n_new == 0 ? 0 : n_valid_host ? n_valid_host[b] : n_new;
    if (n0 < 0 || add < 0 || add > n_new) return TKV_E_INVAL;
    if (n0 + add > d->capacity) return TKV_E_CAPACITY;
    app.app_add.n[b] = add;
  }
  const void* host_dev = nullptr;
  st = tkv::device_view(c->kv_host, tkv::kDevHostOnly, &host_dev);
  if (st != TKV_OK) return st;
  app.app_k = (const __half*)k_new;
  app.app_v = (const __half*)v_new;
  app.app_host = (__half*)host_dev;
  app.app_local = (__half*)c->kv_local;
  app.app_summary = (__half*)c->key_summary;
  app.app_stride = n_new;
  att.att_host = (const __half*)host_dev;
  att.att_local = (const __half*)c->kv_local;
  att.att_out = (__half*)out;
  att.att_scale2 = sm_scale * 1.44269504088896340736f;
  att.pf = (const __half*)next_key_summary;
  // the kernels see the lengths after the append
  for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] += app.app_add.n[b];
  st = estimate_topk_launch(d, c, q, c->key_summary, 0, c->channel_idx, topk_idx, topk_count, workspace,
                            workspace_bytes, stream, nullptr, nullptr, nullptr, n_new > 0 ? &app : nullptr, &att);
  if (st != TKV_OK)
    for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] -= app.app_add.n[b];
  return st;
}
