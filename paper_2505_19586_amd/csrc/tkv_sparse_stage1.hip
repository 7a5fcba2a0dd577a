// Stage 1 of the dynamic retrieval (Sec. 4.2, Fig. 4): per-channel key maxima and a
// channel-major copy of the keys kept up to date on append, the critical channels of Eq. 10,
// and the fetch of the critical key cache for them.  Stage 2 over such a cache is
// tkv_sparse_estimate_topk_cm (tkv_sparse_topk.hip).
#include "tkv_common.h"

namespace {

constexpr int kTile = 64;  // tokens per workgroup of the append kernel

struct Stage1AppendParams {
  float* k_absmax;
  __half* keys_cm;  // device-visible
  const __half* k_new;
  int32_t hkv, capacity, n_stride;
  TkvSeqLens n_old;
  TkvSeqLens n_add;
};

// One workgroup transposes 64 new tokens x 128 channels of one KV head through LDS: every
// channel row of keys_cm receives 64 consecutive tokens (128 contiguous bytes per store
// instruction), and the channel maxima of the tile go to k_absmax with an integer atomic
// maximum (bit patterns of non-negative floats order like integers).
__global__ __launch_bounds__(256) void stage1_append_kernel(Stage1AppendParams p) {
  __shared__ __half tile[kTile][TKV_D + 2];
  const int b = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const int i0 = blockIdx.x * kTile;
  const int add = p.n_add.n[b];
  if (i0 >= add) return;
  const int cnt = min(kTile, add - i0);
  const size_t bh = (size_t)b * p.hkv + h;
  for (int x = tid; x < kTile * (TKV_D / 2); x += 256) {
    const int t = x / (TKV_D / 2), w = x % (TKV_D / 2);
    uint32_t v = 0u;
    if (t < cnt)
      v = reinterpret_cast<const uint32_t*>(p.k_new + (((size_t)b * p.n_stride + i0 + t) * p.hkv + h) * TKV_D)[w];
    *reinterpret_cast<uint32_t*>(&tile[t][2 * w]) = v;
  }
  __syncthreads();
  if (tid < TKV_D) {
    float m = 0.f;
    for (int t = 0; t < cnt; ++t) m = fmaxf(m, fabsf(__half2float(tile[t][tid])));
    atomicMax(reinterpret_cast<uint32_t*>(p.k_absmax + bh * TKV_D + tid), __float_as_uint(m));
  }
  const int lane = tid % 64, wave = tid / 64;
  const size_t tok0 = (size_t)p.n_old.n[b] + i0;
  if (lane < cnt) {
    for (int c = wave; c < TKV_D; c += 4) p.keys_cm[(bh * TKV_D + c) * (size_t)p.capacity + tok0 + lane] = tile[lane][c];
  }
}

struct SelectParams {
  const float* k_absmax;
  const __half* q_hat;
  int32_t* channel_idx;
  int32_t hq, hkv, ds;
};

// One workgroup of 128 threads per (sequence, KV head); thread c owns channel c.
__global__ __launch_bounds__(TKV_D) void select_channels_kernel(SelectParams p) {
  __shared__ float s_s[TKV_D];
  __shared__ uint32_t s_sel[TKV_D];
  const int b = blockIdx.y, h = blockIdx.x;
  const int G = p.hq / p.hkv;
  const size_t bh = (size_t)b * p.hkv + h;
  tkv::select_channels_block(p.q_hat + ((size_t)b * p.hq + (size_t)h * G) * TKV_D, G, p.k_absmax + bh * TKV_D, p.ds,
                             s_s, s_sel, p.channel_idx + bh * p.ds, nullptr);
}

struct PrefetchParams {
  const __half* keys_cm;  // device-visible
  const int32_t* channel_idx;
  __half* keys_out;
  int32_t hkv, ds, capacity;
  TkvSeqLens lens;
};

// Row copies shaped for the host link: one 512-byte piece of a channel row per load
// instruction (64 lanes x 8 bytes), four pieces in flight per wave.
constexpr int kPieces = 4;
__global__ __launch_bounds__(256) void prefetch_rows_kernel(PrefetchParams p) {
  const int b = blockIdx.z, hr = blockIdx.y;  // hr = KV head * d_s + row
  const int h = hr / p.ds, i = hr % p.ds;
  const size_t bh = (size_t)b * p.hkv + h;
  const int n = p.lens.n[b];
  const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  const int ch = p.channel_idx[bh * p.ds + i];
  const __half* src = p.keys_cm + (bh * TKV_D + ch) * (size_t)p.capacity;
  __half* dst = p.keys_out + (bh * p.ds + i) * (size_t)p.capacity;
  const int pieces = (n + 255) / 256;  // 256 tokens = 512 bytes
  constexpr int kPerBlock = 4 * kPieces;
  for (int s0 = blockIdx.x * kPerBlock; s0 < pieces; s0 += gridDim.x * kPerBlock) {
    uint2 v[kPieces];
    int tok[kPieces];
#pragma unroll
    for (int j = 0; j < kPieces; ++j) {
      tok[j] = 256 * (s0 + 4 * j + wave) + 4 * lane;
      // a piece may reach past n, never past the row: capacity is a multiple of 8
      if (tok[j] < n) v[j] = *reinterpret_cast<const uint2*>(src + tok[j]);
    }
#pragma unroll
    for (int j = 0; j < kPieces; ++j)
      if (tok[j] < n) *reinterpret_cast<uint2*>(dst + tok[j]) = v[j];
  }
}

}  // namespace

extern "C" int32_t tkv_sparse_stage1_sizes(const tkv_sparse_desc* d, size_t bytes_out[2]) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!bytes_out) return TKV_E_INVAL;
  const size_t bh = (size_t)d->batch * d->n_kv_heads;
  bytes_out[0] = bh * TKV_D * sizeof(float);
  bytes_out[1] = bh * TKV_D * (size_t)d->capacity * 2;
  return TKV_OK;
}

extern "C" int32_t tkv_sparse_stage1_append(const tkv_sparse_desc* d, const tkv_sparse_cache* c,
                                            const tkv_sparse_stage1* s1, const void* k_new, int32_t n_new,
                                            const int32_t* n_valid_host, void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !s1 || n_new < 0) return TKV_E_INVAL;
  if (d->capacity % 8 != 0) return TKV_E_INVAL;
  if (n_new == 0) return TKV_OK;
  if (!k_new || !s1->k_absmax || !s1->keys_cm) return TKV_E_INVAL;
  Stage1AppendParams p;
  for (int b = 0; b < d->batch; ++b) {
    const int64_t n0 = c->seq_len_host[b];
    const int32_t add = n_valid_host ? n_valid_host[b] : n_new;
    if (n0 < 0 || add < 0 || add > n_new) return TKV_E_INVAL;
    if (n0 + add > d->capacity) return TKV_E_CAPACITY;
    p.n_old.n[b] = (int32_t)n0;
    p.n_add.n[b] = add;
  }
  const void* cm = nullptr;
  st = tkv::device_view(s1->keys_cm, tkv::kDevAny, &cm);
  if (st != TKV_OK) return st;
  p.k_absmax = s1->k_absmax;
  p.keys_cm = (__half*)cm;
  p.k_new = (const __half*)k_new;
  p.hkv = d->n_kv_heads;
  p.capacity = d->capacity;
  p.n_stride = n_new;
  const dim3 grid((n_new + kTile - 1) / kTile, d->n_kv_heads, d->batch);
  TKV_LAUNCH(stage1_append_kernel, grid, 256, 0, (hipStream_t)stream, p);
  return TKV_OK;
}

extern "C" int32_t tkv_sparse_select_channels(const tkv_sparse_desc* d, const tkv_sparse_stage1* s1,
                                              const void* q_hat, int32_t* channel_idx_out, void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!s1 || !s1->k_absmax || !q_hat || !channel_idx_out) return TKV_E_INVAL;
  SelectParams p;
  p.k_absmax = s1->k_absmax;
  p.q_hat = (const __half*)q_hat;
  p.channel_idx = channel_idx_out;
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.ds = d->n_channels;
  TKV_LAUNCH(select_channels_kernel, dim3(d->n_kv_heads, d->batch), TKV_D, 0, (hipStream_t)stream, p);
  return TKV_OK;
}

extern "C" int32_t tkv_sparse_prefetch_keys(const tkv_sparse_desc* d, const tkv_sparse_cache* c,
                                            const tkv_sparse_stage1* s1, const int32_t* channel_idx, void* keys_out,
                                            void* stream) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !s1 || !s1->keys_cm || !channel_idx || !keys_out) return TKV_E_INVAL;
  if (d->capacity % 8 != 0) return TKV_E_INVAL;
  PrefetchParams p;
  int max_n = 0;
  for (int b = 0; b < d->batch; ++b) {
    const int32_t n = c->seq_len_host[b];
    if (n < 0) return TKV_E_INVAL;
    if (n > d->capacity) return TKV_E_CAPACITY;
    p.lens.n[b] = n;
    if (n > max_n) max_n = n;
  }
  if (max_n == 0) return TKV_OK;
  const void* cm = nullptr;
  st = tkv::device_view(s1->keys_cm, tkv::kDevAny, &cm);
  if (st != TKV_OK) return st;
  p.keys_cm = (const __half*)cm;
  p.channel_idx = channel_idx;
  p.keys_out = (__half*)keys_out;
  p.hkv = d->n_kv_heads;
  p.ds = d->n_channels;
  p.capacity = d->capacity;
  // about 1024 workgroups over the whole launch, each covering 16 pieces per pass
  const int rows = d->n_kv_heads * d->n_channels * d->batch;
  const int pieces = (max_n + 255) / 256;
  int gx = (1024 + rows - 1) / rows;
  const int gx_max = (pieces + 15) / 16;
  if (gx > gx_max) gx = gx_max;
  if (gx < 1) gx = 1;
  TKV_LAUNCH(prefetch_rows_kernel, dim3(gx, d->n_kv_heads * d->n_channels, d->batch), 256, 0, (hipStream_t)stream, p);
  return TKV_OK;
}
