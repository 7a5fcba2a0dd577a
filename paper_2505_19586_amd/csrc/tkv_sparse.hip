// Sparsity-friendly layers (Sec. 4.2): cache update, fetch of the selected rows from
// pinned host memory, exact attention over n_local + n_topk tokens (Sec. 5.1).
// Scoring and Top-K live in tkv_sparse_topk.hip.
#include "tkv_common.h"

namespace {

// ---------------------------------------------------------------------------------

struct AppendParams {
  __half* summary;
  const int32_t* channel_idx;
  __half* kv_host;
  __half* kv_local;
  const __half* k_new;
  const __half* v_new;
  float* k_absmax;   // Stage 1 buffers updated by the same launch (short appends), or null
  __half* keys_cm;
  int32_t hkv, ds, n_sink, n_window, capacity;
  int32_t n_stride;  // rows per sequence in k_new / v_new
  TkvSeqLens n_old;
  TkvSeqLens n_add;  // valid new rows per sequence
};

// One workgroup per new token up to kAppendGrid workgroups per sequence, which then walk the
// tokens with the grid's stride: a bulk append (prefill) is bound by the device-to-host link,
// and a launch that is no wider than the link needs leaves the rest of the machine to the
// kernels of other streams (the next layers' computation) instead of parking tens of thousands
// of workgroups that wait for the link on every compute unit.
constexpr int kAppendGrid = 1024;
__global__ __launch_bounds__(256) void sparse_append_kernel(AppendParams p) {
  const int b = blockIdx.y, tid = threadIdx.x;
  for (int i = blockIdx.x; i < p.n_add.n[b]; i += gridDim.x) {
  const int n0 = p.n_old.n[b], n1 = n0 + p.n_add.n[b];
  const int tok = n0 + i;
  const int chunks = p.hkv * 16;
  const bool local = tok < p.n_sink || tok >= n1 - p.n_window;
  const int slot = tok < p.n_sink ? tok : p.n_sink + tok % p.n_window;
  for (int x = tid; x < 2 * chunks; x += 256) {
    const int kv = x / chunks, rem = x % chunks, h = rem / 16, part = rem % 16;
    const size_t bh = (size_t)b * p.hkv + h;
    const uint4 v = reinterpret_cast<const uint4*>((kv ? p.v_new : p.k_new) +
                                                   (((size_t)b * p.n_stride + i) * p.hkv + h) * TKV_D)[part];
    reinterpret_cast<uint4*>(p.kv_host + ((bh * p.capacity + tok) * 2 + kv) * TKV_D)[part] = v;
    if (local)
      reinterpret_cast<uint4*>(p.kv_local + ((bh * (p.n_sink + p.n_window) + slot) * 2 + kv) * TKV_D)[part] = v;
  }
  for (int x = tid; x < p.hkv * p.ds; x += 256) {
    const int h = x / p.ds, ci = x % p.ds;
    const size_t bh = (size_t)b * p.hkv + h;
    const int c = p.channel_idx[bh * p.ds + ci];
    p.summary[(bh * p.capacity + tok) * p.ds + ci] = p.k_new[(((size_t)b * p.n_stride + i) * p.hkv + h) * TKV_D + c];
  }
  if (p.keys_cm != nullptr) {
    // Stage 1 (Sec. 4.2): the token's column of the channel-major keys and the running maxima
    // of Eq. 10 (bit patterns of non-negative floats order like integers)
    for (int x = tid; x < p.hkv * TKV_D; x += 256) {
      const int h = x / TKV_D, c = x % TKV_D;
      const size_t bh = (size_t)b * p.hkv + h;
      const __half v = p.k_new[(((size_t)b * p.n_stride + i) * p.hkv + h) * TKV_D + c];
      p.keys_cm[(bh * TKV_D + c) * (size_t)p.capacity + tok] = v;
      atomicMax(reinterpret_cast<uint32_t*>(p.k_absmax + bh * TKV_D + c), __float_as_uint(fabsf(__half2float(v))));
    }
  }
  }
}

// ---------------------------------------------------------------------------------

struct GatherParams {
  const __half* kv_host;  // device-visible address of the pinned host cache
  const int32_t* topk_idx;
  const int32_t* topk_count;
  __half* staging;
  int32_t hkv, top_k, capacity;
};

// One 64-lane wave moves one 512-byte row (K row + V row of a token) with a single 8-byte
// load per lane straight from pinned host memory: one whole row per load instruction is the
// request shape that the host link serves fastest (16-byte lanes, i.e. two rows per
// instruction, measured 25 % slower).  Every wave keeps four rows in flight and walks the
// rows with the stride of the grid, which is sized to a quarter of the machine's wave slots:
// the transfer rate is the same as with one row per wave, and kernels of other streams can
// run beside it.
constexpr int kGatherRows = 4;  // rows in flight per wave
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherParams p) {
  const int b = blockIdx.z, h = blockIdx.y;
  const size_t bh = (size_t)b * p.hkv + h;
  // (count and indices are the caller's data: kept inside the buffers whatever they hold)
  const int cnt = min(max(p.topk_count[bh], 0), p.top_k);
  const int part = threadIdx.x % 64, wave = threadIdx.x / 64;
  constexpr int kPerBlock = 4 * kGatherRows;
  for (int r0 = blockIdx.x * kPerBlock; r0 < cnt; r0 += gridDim.x * kPerBlock) {
    uint2 v[kGatherRows];
#pragma unroll
    for (int j = 0; j < kGatherRows; ++j) {
      const int row = min(r0 + 4 * j + wave, cnt - 1);
      const int tok = min(max(p.topk_idx[bh * p.top_k + row], 0), p.capacity - 1);
      v[j] = reinterpret_cast<const uint2*>(p.kv_host + (bh * p.capacity + (size_t)tok) * 2 * TKV_D)[part];
    }
#pragma unroll
    for (int j = 0; j < kGatherRows; ++j) {
      const int row = r0 + 4 * j + wave;
      if (row < cnt) reinterpret_cast<uint2*>(p.staging + (bh * p.top_k + (size_t)row) * 2 * TKV_D)[part] = v[j];
    }
  }
}

struct SparseAttnParams {
  const __half* q;
  const __half* staging;
  const __half* kv_host;    // fused variant: device-visible view of the pinned host rows
  const int32_t* topk_idx;  // fused variant
  int32_t capacity;
  uint32_t* arrivals;  // [B][Hkv] stride 8 words, zero between calls
  __half* out;         // [B][Hq][D]
  const __half* kv_local;
  const int32_t* topk_count;
  float* parts;
  float scale2;
  int32_t hq, hkv, top_k, n_sink, n_window, n_chunks;
  TkvSeqLens lens;
};

constexpr int kAttnMaxWaves = 4;  // a workgroup of W waves handles 32*W attended tokens

__device__ inline float half_wave_max(float v) {
  for (int m = 16; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

constexpr int kRowPitch = 2 * TKV_D * 2 + 16;  // LDS bytes per staged K|V row (padded against bank conflicts)

// Exact attention over sinks + gathered rows + window.  One workgroup of W <= 4 waves
// handles 32*W attended tokens of one KV head; lane (t, hp) scores token t for the query heads
// [GH/2 hp, GH/2 hp + GH/2) of the group (GH = 4, or 8 for groups of 5 to 8 heads); then every
// lane accumulates two output channels of all heads.
// FUSED: the selected rows are not read from the staging buffer but fetched by this kernel
// from pinned host memory (one 512-byte row per load instruction, all 32 rows of a wave in
// flight) into LDS, so the transfer and the attention are one launch.
template <bool FUSED, int GH>
__global__ __launch_bounds__(256) void sparse_attn_kernel(SparseAttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char rows_s[];  // FUSED: [W][32][kRowPitch]
  constexpr int HPH = GH / 2;  // heads per half-wave
  __shared__ const __half* src_s[4][32];
  __shared__ float qs[GH][TKV_D];
  __shared__ float pw[4][GH][32];
  __shared__ const __half* vrow_s[4][32];
  __shared__ float red_m[4][GH], red_l[4][GH];
  __shared__ float red_o[4][GH][TKV_D];
  const int b = blockIdx.z, h = blockIdx.y, chunk = blockIdx.x;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int G = p.hq / p.hkv;
  const size_t bh = (size_t)b * p.hkv + h;
  const int n = p.lens.n[b];
  const int n_sk = min(p.n_sink, n);
  const int cnt = min(max(p.topk_count[bh], 0), p.top_k);  // (the caller's data: kept inside the buffers)
  const int w0 = max(n - p.n_window, n_sk);
  const int n_att = n_sk + cnt + (n - w0);

  const int nthr = blockDim.x, W = nthr / 64;
  for (int i = tid; i < GH * TKV_D; i += nthr) {
    const int hh = i / TKV_D, c = i % TKV_D;
    qs[hh][c] = hh < G ? __half2float(p.q[((size_t)b * p.hq + (size_t)h * G + hh) * TKV_D + c]) : 0.f;
  }
  __syncthreads();

  const int t = lane % 32, hp = lane / 32;
  const int i = (chunk * W + wave) * 32 + t;
  const bool valid = i < n_att;
  // invalid tokens point at a real row and carry weight 0, so no loop needs a branch
  const __half* krow = p.kv_local + bh * (size_t)(p.n_sink + p.n_window) * 2 * TKV_D;
  if (valid) {
    if (i < n_sk)
      krow = p.kv_local + (bh * (p.n_sink + p.n_window) + i) * 2 * TKV_D;
    else if (i < n_sk + cnt) {
      if (FUSED) {
        const int tok = min(max(p.topk_idx[bh * p.top_k + (i - n_sk)], 0), p.capacity - 1);
        krow = p.kv_host + (bh * p.capacity + (size_t)tok) * 2 * TKV_D;
      } else {
        krow = p.staging + (bh * p.top_k + (size_t)(i - n_sk)) * 2 * TKV_D;
      }
    } else {
      const int tok = w0 + (i - n_sk - cnt);
      krow = p.kv_local + (bh * (p.n_sink + p.n_window) + p.n_sink + tok % p.n_window) * 2 * TKV_D;
    }
  }
  if (FUSED) {
    // every row of this wave (host or device memory alike): 64 lanes x 8 bytes per row
    unsigned char* rows = rows_s + (size_t)wave * 32 * kRowPitch;
    if (hp == 0) src_s[wave][t] = krow;
    uint2 r[32];
#pragma unroll
    for (int y = 0; y < 32; ++y) r[y] = reinterpret_cast<const uint2*>(src_s[wave][y])[lane];
#pragma unroll
    for (int y = 0; y < 32; ++y) *reinterpret_cast<uint2*>(rows + y * kRowPitch + 8 * lane) = r[y];
    krow = reinterpret_cast<const __half*>(rows + t * kRowPitch);
  }
  float xs[HPH];
#pragma unroll
  for (int y = 0; y < HPH; ++y) xs[y] = -INFINITY;
  if (valid) {
    float a[HPH];
#pragma unroll
    for (int y = 0; y < HPH; ++y) a[y] = 0.f;
    for (int c8 = 0; c8 < TKV_D / 8; ++c8) {
      union {
        uint4 v;
        __half hx[8];
      } u;
      u.v = reinterpret_cast<const uint4*>(krow)[c8];
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const float kx = __half2float(u.hx[x]);
#pragma unroll
        for (int y = 0; y < HPH; ++y) a[y] += qs[HPH * hp + y][c8 * 8 + x] * kx;
      }
    }
#pragma unroll
    for (int y = 0; y < HPH; ++y) xs[y] = a[y] * p.scale2;
  }
  bool any = false;  // this wave has at least one valid token (uniform per wave)
#pragma unroll
  for (int y = 0; y < HPH; ++y) {
    const float m = half_wave_max(xs[y]);
    any = m != -INFINITY;
    pw[wave][HPH * hp + y][t] = valid ? exp2f(xs[y] - m) : 0.f;
    if (t == 0) red_m[wave][HPH * hp + y] = m;
  }
  if (hp == 0) vrow_s[wave][t] = krow + TKV_D;
  __syncthreads();
  const int c0 = 2 * lane;
  float o0[GH], o1[GH], ls[GH];
#pragma unroll
  for (int hh = 0; hh < GH; ++hh) o0[hh] = 0.f, o1[hh] = 0.f, ls[hh] = 0.f;
  if (any) {
#pragma unroll
    for (int t8 = 0; t8 < 32; t8 += 8) {
      __half2 v2[8];
#pragma unroll
      for (int y = 0; y < 8; ++y) v2[y] = reinterpret_cast<const __half2*>(vrow_s[wave][t8 + y])[lane];
#pragma unroll
      for (int y = 0; y < 8; ++y) {
        const float v0 = __low2float(v2[y]), v1 = __high2float(v2[y]);
#pragma unroll
        for (int hh = 0; hh < GH; ++hh) {
          const float pp = pw[wave][hh][t8 + y];
          o0[hh] += pp * v0;
          o1[hh] += pp * v1;
          ls[hh] += pp;
        }
      }
    }
  }
  for (int hh = 0; hh < GH; ++hh) {
    red_o[wave][hh][c0] = o0[hh];
    red_o[wave][hh][c0 + 1] = o1[hh];
    if (lane == 0) red_l[wave][hh] = ls[hh];
  }
  __syncthreads();
  for (int x = tid; x < G * TKV_D; x += nthr) {
    const int hh = x / TKV_D, c = x % TKV_D;
    float M = -INFINITY;
    for (int w = 0; w < W; ++w) M = fmaxf(M, red_m[w][hh]);
    float L = 0.f, O = 0.f;
    for (int w = 0; w < W; ++w) {
      const float mw = red_m[w][hh];
      const float wgt = mw == -INFINITY ? 0.f : exp2f(mw - M);
      L += red_l[w][hh] * wgt;
      O += red_o[w][hh][c] * wgt;
    }
    float* dst = p.parts + (((size_t)b * p.hq + (size_t)h * G + hh) * p.n_chunks + chunk) * TKV_PART_STRIDE;
    // device-scope stores: visible to the merging workgroup without a cache write-back
    __hip_atomic_store(dst + TKV_PART_O + c, O, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (c == 0) {
      __hip_atomic_store(dst, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(dst + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  // ---- the last workgroup of this (sequence, KV head) to arrive merges all chunks; the
  // partials are ordered before the arrival counter by waiting for the stores to complete
  __shared__ uint32_t s_last;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  uint32_t* arrive = p.arrivals + bh * 8 + 4;
  if (tid == 0) s_last = atomicAdd(arrive, 1u) == (uint32_t)(p.n_chunks - 1) ? 1u : 0u;
  __syncthreads();
  if (s_last == 0u) return;
  if (tid == 0) __hip_atomic_store(arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __shared__ float merge_s[3 * 4 * 64 + 4 * 4 * TKV_D + 4];
  const float* head0 = p.parts + ((size_t)b * p.hq + (size_t)h * G) * p.n_chunks * TKV_PART_STRIDE;
  if (nthr >= 64 * min(G, 4)) {
    // (four heads at a time: the merge's LDS scratch is laid out for that many)
    for (int g0 = 0; g0 < G; g0 += 4) {
      if (g0 > 0) __syncthreads();
      tkv::merge_chunks(head0 + (size_t)g0 * p.n_chunks * TKV_PART_STRIDE, min(4, G - g0), p.n_chunks,
                        p.out + ((size_t)b * p.hq + (size_t)h * G + g0) * TKV_D, merge_s, tid, nthr);
    }
  } else {  // one-wave workgroups (few attended tokens): plain loop over the chunks
    auto ld = [](const float* ptr) { return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    for (int x = tid; x < G * TKV_D; x += nthr) {
      const int hh = x / TKV_D, c = x % TKV_D;
      const float* base = head0 + (size_t)hh * p.n_chunks * TKV_PART_STRIDE;
      float M = -INFINITY;
      for (int k = 0; k < p.n_chunks; ++k) M = fmaxf(M, ld(base + (size_t)k * TKV_PART_STRIDE));
      float L = 0.f, O = 0.f;
      for (int k = 0; k < p.n_chunks; ++k) {
        const float* pk = base + (size_t)k * TKV_PART_STRIDE;
        const float mk = ld(pk);
        const float w = mk == -INFINITY ? 0.f : exp2f(mk - M);
        L = __builtin_fmaf(ld(pk + 1), w, L);
        O = __builtin_fmaf(ld(pk + TKV_PART_O + c), w, O);
      }
      p.out[((size_t)b * p.hq + (size_t)h * G + hh) * TKV_D + c] = __float2half_rn(L > 0.f ? O / L : 0.f);
    }
  }
}

int32_t fill_lens(const tkv_sparse_desc* d, const tkv_sparse_cache* c, TkvSeqLens& lens, int& max_n) {
  max_n = 0;
  for (int b = 0; b < d->batch; ++b) {
    const int32_t n = c->seq_len_host[b];
    if (n < 0) return TKV_E_INVAL;
    if (n > d->capacity) return TKV_E_CAPACITY;
    lens.n[b] = n;
    if (n > max_n) max_n = n;
  }
  return TKV_OK;
}

}  // namespace

namespace {
constexpr int kFusedStage1Rows = 8;  // appends up to this long update the Stage 1 buffers in the same launch
}

extern "C" int32_t tkv_sparse_append_dynamic(const tkv_sparse_desc* d, tkv_sparse_cache* c,
                                             const tkv_sparse_stage1* s1, const void* k_new, const void* v_new,
                                             int32_t n_new, const int32_t* n_valid_host, void* stream) {
  if (s1 != nullptr && n_new > kFusedStage1Rows) {
    // long appends: the tiled transpose kernel first, then the plain append
    const int32_t st1 = tkv_sparse_stage1_append(d, c, s1, k_new, n_new, n_valid_host, stream);
    if (st1 != TKV_OK) return st1;
    s1 = nullptr;
  }
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || n_new < 0) return TKV_E_INVAL;
  if (n_new == 0) return TKV_OK;
  if (!k_new || !v_new || !c->key_summary || !c->channel_idx || !c->kv_host || !c->kv_local) return TKV_E_INVAL;
  AppendParams p;
  for (int b = 0; b < d->batch; ++b) {
    const int64_t n0 = c->seq_len_host[b];
    const int32_t add = n_valid_host ? n_valid_host[b] : n_new;
    if (n0 < 0 || add < 0 || add > n_new) return TKV_E_INVAL;
    if (n0 + add > d->capacity) return TKV_E_CAPACITY;
    p.n_old.n[b] = (int32_t)n0;
    p.n_add.n[b] = add;
  }
  const void* host_dev = nullptr;
  st = tkv::device_view(c->kv_host, tkv::kDevHostOnly, &host_dev);
  if (st != TKV_OK) return st;
  p.summary = (__half*)c->key_summary;
  p.channel_idx = c->channel_idx;
  p.kv_host = (__half*)host_dev;
  p.kv_local = (__half*)c->kv_local;
  p.k_new = (const __half*)k_new;
  p.v_new = (const __half*)v_new;
  p.k_absmax = nullptr;
  p.keys_cm = nullptr;
  if (s1 != nullptr) {
    if (!s1->k_absmax || !s1->keys_cm) return TKV_E_INVAL;
    const void* cm = nullptr;
    st = tkv::device_view(s1->keys_cm, tkv::kDevAny, &cm);
    if (st != TKV_OK) return st;
    p.k_absmax = s1->k_absmax;
    p.keys_cm = (__half*)cm;
  }
  p.hkv = d->n_kv_heads;
  p.ds = d->n_channels;
  p.n_sink = d->n_sink;
  p.n_window = d->n_window;
  p.capacity = d->capacity;
  p.n_stride = n_new;
  TKV_LAUNCH(sparse_append_kernel, dim3(n_new < kAppendGrid ? n_new : kAppendGrid, d->batch), 256, 0, (hipStream_t)stream, p);
  for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] += p.n_add.n[b];
  return TKV_OK;
}

extern "C" int32_t tkv_sparse_append_ragged(const tkv_sparse_desc* d, tkv_sparse_cache* c, const void* k_new,
                                            const void* v_new, int32_t n_new, const int32_t* n_valid_host,
                                            void* stream) {
  return tkv_sparse_append_dynamic(d, c, nullptr, k_new, v_new, n_new, n_valid_host, stream);
}

extern "C" int32_t tkv_sparse_append(const tkv_sparse_desc* d, tkv_sparse_cache* c, const void* k_new,
                                     const void* v_new, int32_t n_new, void* stream) {
  return tkv_sparse_append_ragged(d, c, k_new, v_new, n_new, nullptr, stream);
}

extern "C" int32_t tkv_sparse_gather(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const int32_t* topk_idx,
                                     const int32_t* topk_count, void* staging, void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->kv_host || !topk_idx || !topk_count || !staging) return TKV_E_INVAL;
  const void* host_dev = nullptr;
  st = tkv::device_view(c->kv_host, tkv::kDevHostOnly, &host_dev);
  if (st != TKV_OK) return st;
  GatherParams p;
  p.kv_host = (const __half*)host_dev;
  p.topk_idx = topk_idx;
  p.topk_count = topk_count;
  p.staging = (__half*)staging;
  p.hkv = d->n_kv_heads;
  p.top_k = d->top_k;
  p.capacity = d->capacity;
  // about 512 workgroups in total, never more per head than there are rows to move
  int gx = (512 + d->n_kv_heads * d->batch - 1) / (d->n_kv_heads * d->batch);
  const int gmax = (d->top_k + 4 * kGatherRows - 1) / (4 * kGatherRows);
  if (gx > gmax) gx = gmax;
  if (gx < 1) gx = 1;
  TKV_LAUNCH(gather_rows_kernel, dim3(gx, d->n_kv_heads, d->batch), 256, 0, (hipStream_t)stream, p);
  return TKV_OK;
}

namespace tkv {
// tkv_sparse_topk.hip: the one-launch step's fetch + attention phase for a selection made earlier
int32_t launch_fetch_attn(const tkv_sparse_desc* d, const TkvSeqLens& lens, const __half* q, const int32_t* topk_idx,
                          const int32_t* topk_count, const __half* host_rows, const __half* local_rows, __half* out,
                          float scale2, hipStream_t s);
}  // namespace tkv

namespace {
// Attention over sinks + selected rows + window.  topk_idx_fused == nullptr: the selected
// rows are in `staging`; otherwise they are fetched from the pinned host cache by the
// attention kernel itself.
int32_t sparse_attn_launch(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const void* q,
                           const int32_t* topk_idx_fused, const int32_t* topk_count, const void* staging, void* out,
                           float sm_scale, void* workspace, size_t workspace_bytes, void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !c->kv_local || !q || !topk_count || !out || !workspace) return TKV_E_INVAL;
  size_t need = 0;
  tkv_sparse_cache_sizes(d, nullptr, &need);
  if (workspace_bytes < need) return TKV_E_WORKSPACE;
  SparseAttnParams p;
  int max_n = 0;
  st = fill_lens(d, c, p.lens, max_n);
  if (st != TKV_OK) return st;
  const int max_att = d->n_sink + d->top_k + d->n_window;
  // four waves per workgroup once there is work for them: few chunks keep the final merge
  // short (and their number must stay within the 64 partial slots)
  int W = max_att > 256 ? kAttnMaxWaves : 1;
  const int n_chunks = (max_att + 32 * W - 1) / (32 * W);
  if (n_chunks > 64) return TKV_E_UNSUPPORTED;
  // partials live behind the Top-K scratch so that one workspace serves both calls
  float* parts = tkv::carve_sparse_ws(d, workspace).parts;
  p.q = (const __half*)q;
  p.staging = (const __half*)staging;
  p.kv_local = (const __half*)c->kv_local;
  p.topk_count = topk_count;
  p.parts = parts;
  p.scale2 = sm_scale * 1.44269504088896340736f;
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.top_k = d->top_k;
  p.n_sink = d->n_sink;
  p.n_window = d->n_window;
  p.n_chunks = n_chunks;
  hipStream_t s = (hipStream_t)stream;
  const bool big_group = d->n_q_heads / d->n_kv_heads > 4;  // 5 to 8 query heads per KV head
  p.kv_host = nullptr;
  p.topk_idx = nullptr;
  p.capacity = d->capacity;
  p.arrivals = tkv::carve_sparse_ws(d, workspace).ctrl;  // word 4 of each head's 8 control words
  p.out = (__half*)out;
  if (topk_idx_fused) {
    const void* host_dev = nullptr;
    st = tkv::device_view(c->kv_host, tkv::kDevHostOnly, &host_dev);
    if (st != TKV_OK) return st;
    p.kv_host = (const __half*)host_dev;
    p.topk_idx = topk_idx_fused;
    // Groups of up to 4 query heads: one workgroup per head whose 16 waves keep two passes of
    // rows in flight each (the attention phase of tkv_sparse_decode): the link-bound loop without
    // a cross-workgroup merge behind it.
    st = tkv::launch_fetch_attn(d, p.lens, p.q, topk_idx_fused, topk_count, p.kv_host, p.kv_local, p.out, p.scale2, s);
    if (st != TKV_E_UNSUPPORTED) return st;
    static const bool lds_ok =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&sparse_attn_kernel<true, 4>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kAttnMaxWaves * 32 * kRowPitch) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(&sparse_attn_kernel<true, 8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kAttnMaxWaves * 32 * kRowPitch) == hipSuccess;
    if (!lds_ok) return TKV_E_HIP;
    const dim3 grid(n_chunks, d->n_kv_heads, d->batch);
    if (big_group) {
      TKV_LAUNCH((sparse_attn_kernel<true, 8>), grid, 64 * W, W * 32 * kRowPitch, s, p);
    } else {
      TKV_LAUNCH((sparse_attn_kernel<true, 4>), grid, 64 * W, W * 32 * kRowPitch, s, p);
    }
  } else if (big_group) {
    TKV_LAUNCH((sparse_attn_kernel<false, 8>), dim3(n_chunks, d->n_kv_heads, d->batch), 64 * W, 0, s, p);
  } else {
    TKV_LAUNCH((sparse_attn_kernel<false, 4>), dim3(n_chunks, d->n_kv_heads, d->batch), 64 * W, 0, s, p);
  }
  return TKV_OK;
}
}  // namespace

extern "C" int32_t tkv_sparse_attn(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const void* q,
                                   const int32_t* topk_count, const void* staging, void* out, float sm_scale,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  if (!staging) return TKV_E_INVAL;
  return sparse_attn_launch(d, c, q, nullptr, topk_count, staging, out, sm_scale, workspace, workspace_bytes, stream);
}

namespace {
// Two events per host thread order the gather stream against the compute stream.  They carry
// no data; re-recording an event only affects waits enqueued later, and a thread enqueues its
// record / wait pairs in program order, so calls of different threads (on their own streams)
// cannot pick up each other's records.
struct StreamLink {
  hipEvent_t topk_ready = nullptr, rows_ready = nullptr;
  int32_t init() {
    if (topk_ready) return TKV_OK;
    if (hipEventCreateWithFlags(&topk_ready, hipEventDisableTiming) != hipSuccess) return TKV_E_HIP;
    if (hipEventCreateWithFlags(&rows_ready, hipEventDisableTiming) != hipSuccess) return TKV_E_HIP;
    return TKV_OK;
  }
};
thread_local StreamLink g_link;
}  // namespace

extern "C" int32_t tkv_sparse_gather_attn(const tkv_sparse_desc* d, const tkv_sparse_cache* c, const void* q,
                                          const int32_t* topk_idx, const int32_t* topk_count, void* out,
                                          float sm_scale, void* staging, void* workspace, size_t workspace_bytes,
                                          void* gather_stream, void* compute_stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !c->kv_local || !c->kv_host || !q || !topk_idx || !topk_count || !staging || !out ||
      !workspace)
    return TKV_E_INVAL;
  size_t need = 0;
  tkv_sparse_cache_sizes(d, nullptr, &need);
  if (workspace_bytes < need) return TKV_E_WORKSPACE;
  hipStream_t gs = (hipStream_t)gather_stream, cs = (hipStream_t)compute_stream;
  const bool two = gs != cs;
  // one stream: nothing can overlap, so the attention kernel fetches the rows itself
  if (!two)
    return sparse_attn_launch(d, c, q, topk_idx, topk_count, staging, out, sm_scale, workspace, workspace_bytes, cs);
  if (two) {
    if (g_link.init() != TKV_OK) return TKV_E_HIP;
    TKV_HIP_TRY(hipEventRecord(g_link.topk_ready, cs));
    TKV_HIP_TRY(hipStreamWaitEvent(gs, g_link.topk_ready, 0));
  }
  st = tkv_sparse_gather(d, c, topk_idx, topk_count, staging, gs);
  if (st != TKV_OK) return st;
  if (two) {
    TKV_HIP_TRY(hipEventRecord(g_link.rows_ready, gs));
    TKV_HIP_TRY(hipStreamWaitEvent(cs, g_link.rows_ready, 0));
  }
  return tkv_sparse_attn(d, c, q, topk_count, staging, out, sm_scale, workspace, workspace_bytes, cs);
}
