// Offline identification (Sec. 4.1): dense preference score of a layer, Eq. 6-8, and the
// classification of Eq. 9.  Per KV head: the attention logits of the n_q most recent queries
// of its query heads against all n keys (a dense contraction: MFMA), the exact Top-K of every
// logit row (the selection kernels of the sparse path, run on the logits) and the mass of
// the selected entries under the row's softmax.
#include "tkv_common.h"

namespace tkv {
int32_t topk_of_scores(const float* scores, size_t stride, int n_rows, int n, int top_k, int capacity, SparseWs ws,
                       int32_t* topk_idx, int32_t* topk_count, hipStream_t s);
}

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kTokBlock = 512;  // tokens per workgroup of the logits kernel

struct PrefParams {
  const __half* q_last;  // [B][n_q][Hq][128]
  const __half* k;       // [B][n][Hkv][128]
  float* scores;         // [R][stride]: row r = (query head of the group) * n_q + position, log2 units
  float* ml;             // [R][ntb][2]: per token block, row maximum and sum of 2^(x - max)
  const int32_t* topk_idx;
  const int32_t* topk_count;
  float* row_p;          // [R]: 1 - top-k mass of every row
  float* p_out;          // [B][Hq]
  float scale2;          // sm_scale * log2(e)
  int32_t hq, hkv, n_q, n, b, h, ntb, top_k;
  size_t stride;
};

// merge of two (maximum, sum) pairs of a softmax in log2 units
__device__ inline void ml_merge(float& m, float& l, float m2, float l2) {
  const float mn = fmaxf(m, m2);
  const float a = m == -INFINITY ? 0.f : exp2f(m - mn), b = m2 == -INFINITY ? 0.f : exp2f(m2 - mn);
  l = l * a + l2 * b;
  m = mn;
}

// One wave = one tile of 16 query rows against the workgroup's 512 tokens, 16 tokens per
// v_mfma_f32_16x16x32_f16 column tile (A = query rows, B = key rows, both read straight from
// global memory in operand order: 16 bytes per lane and 32-channel slab).
__global__ __launch_bounds__(256) void pref_logits_kernel(PrefParams p) {
  const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  const int G = p.hq / p.hkv, R = G * p.n_q;
  const int rt = 4 * blockIdx.y + wave;  // row tile of this wave
  if (16 * rt >= R) return;
  const int r0 = 16 * rt;
  const int col = lane % 16, kb = lane / 16;
  // A operand: row r0 + col of the group = query head j, position i
  uintx4 a[4];
  {
    const int r = r0 + col, j = r / p.n_q, i = r % p.n_q;
    const __half* qrow = p.q_last + (((size_t)p.b * p.n_q + i) * p.hq + (size_t)p.h * G + j) * TKV_D;
#pragma unroll
    for (int m = 0; m < 4; ++m) a[m] = *reinterpret_cast<const uintx4*>(qrow + 32 * m + 8 * kb);
  }
  float mx[4], ls[4];
#pragma unroll
  for (int x = 0; x < 4; ++x) mx[x] = -INFINITY, ls[x] = 0.f;
  const int t_blk = blockIdx.x * kTokBlock;
  for (int t0 = t_blk; t0 < min(t_blk + kTokBlock, p.n); t0 += 16) {
    const int t = t0 + col;
    const int tc = min(t, p.n - 1);  // columns past the end re-read the last key and are dropped
    const __half* krow = p.k + (((size_t)p.b * p.n + tc) * p.hkv + p.h) * TKV_D;
    uintx4 bk[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) bk[m] = *reinterpret_cast<const uintx4*>(krow + 32 * m + 8 * kb);
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < 4; ++m)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a[m]), __builtin_bit_cast(half8, bk[m]),
                                                   acc, 0, 0, 0);
    // this lane holds rows r0 + 4 kb + x of token t
    if (t < p.n) {
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const float v = acc[x] * p.scale2;
        p.scores[(size_t)(r0 + 4 * kb + x) * p.stride + t] = v;
        const float mn = fmaxf(mx[x], v);
        ls[x] = ls[x] * exp2f(mx[x] - mn) + exp2f(v - mn);  // exp2f(-inf) = 0 on the first token
        mx[x] = mn;
      }
    }
  }
  // rows are spread over the 16 lanes with the same kb: merge them
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    for (int d = 1; d < 16; d <<= 1) {
      const float m2 = __shfl_xor(mx[x], d, 64), l2 = __shfl_xor(ls[x], d, 64);
      ml_merge(mx[x], ls[x], m2, l2);
    }
    if (col == 0) {
      float* dst = p.ml + ((size_t)(r0 + 4 * kb + x) * p.ntb + blockIdx.x) * 2;
      dst[0] = mx[x];
      dst[1] = ls[x];
    }
  }
}

__device__ inline float block_sum(float v, float* scratch) {
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  __syncthreads();
  if (threadIdx.x % 64 == 0) scratch[threadIdx.x / 64] = v;
  __syncthreads();
  return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

// One workgroup per query row: its share of Eq. 8 (1 - mass of the selected keys) from the
// row's softmax statistics and the logits of the selected keys.
__global__ __launch_bounds__(256) void pref_row_kernel(PrefParams p) {
  __shared__ float scratch[4];
  __shared__ float s_m[4], s_l[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  float m = -INFINITY, l = 0.f;
  for (int tb = tid; tb < p.ntb; tb += 256) {
    const float* src = p.ml + ((size_t)r * p.ntb + tb) * 2;
    ml_merge(m, l, src[0], src[1]);
  }
  for (int d = 32; d >= 1; d >>= 1) {
    const float m2 = __shfl_xor(m, d, 64), l2 = __shfl_xor(l, d, 64);
    ml_merge(m, l, m2, l2);
  }
  if (tid % 64 == 0) s_m[tid / 64] = m, s_l[tid / 64] = l;
  __syncthreads();
  m = s_m[0], l = s_l[0];
  for (int w = 1; w < 4; ++w) ml_merge(m, l, s_m[w], s_l[w]);
  const int cnt = p.topk_count[r];
  float tsum = 0.f;
  for (int e = tid; e < cnt; e += 256) {
    const int t = p.topk_idx[(size_t)r * p.top_k + e];
    tsum += exp2f(p.scores[(size_t)r * p.stride + t] - m);
  }
  tsum = block_sum(tsum, scratch);
  if (tid == 0) p.row_p[r] = l > 0.f ? 1.0f - tsum / l : 0.f;
}

// Eq. 8 per query head: the sum of its rows' shares, in row order (one thread per head).
__global__ void pref_sum_kernel(PrefParams p) {
  const int j = threadIdx.x;
  const int G = p.hq / p.hkv;
  if (j >= G) return;
  float total = 0.f;
  for (int i = 0; i < p.n_q; ++i) total += p.row_p[j * p.n_q + i];
  p.p_out[(size_t)p.b * p.hq + (size_t)p.h * G + j] = total;
}

int32_t check_pref_desc(const tkv_pref_desc* d) {
  if (!d || d->struct_size != sizeof(tkv_pref_desc)) return TKV_E_INVAL;
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->batch <= 0 || d->n_q <= 0 || d->top_k <= 0 || d->capacity <= 0)
    return TKV_E_INVAL;
  if (d->n_q_heads % d->n_kv_heads != 0) return TKV_E_INVAL;
  if (d->head_dim != TKV_D || d->batch > TKV_MAX_BATCH) return TKV_E_UNSUPPORTED;
  const int g = d->n_q_heads / d->n_kv_heads;
  if (g != 1 && g != 2 && g != 4) return TKV_E_UNSUPPORTED;
  if (d->n_q % 16 != 0 || d->n_q > 256 || d->top_k > 4096) return TKV_E_UNSUPPORTED;
  return TKV_OK;
}

// Workspace carve-up for one (sequence, KV head) at a time: logits, softmax partials, Top-K
// output, then the selection workspace of R "heads".
struct PrefWs {
  float* scores;
  float* ml;
  int32_t* topk_idx;
  int32_t* topk_count;
  float* row_p;
  void* select_ws;
  size_t stride;
  int32_t ntb;
  tkv_sparse_desc sel;  // descriptor the selection workspace is laid out for
};
size_t pref_ws_layout(const tkv_pref_desc* d, char* base, PrefWs* out) {
  const size_t R = (size_t)(d->n_q_heads / d->n_kv_heads) * d->n_q;
  const size_t stride = ((size_t)d->capacity + 63) & ~(size_t)63;
  const int32_t ntb = (d->capacity + kTokBlock - 1) / kTokBlock;
  tkv_sparse_desc sel = {};
  sel.struct_size = sizeof(tkv_sparse_desc);
  sel.n_q_heads = (int32_t)R;
  sel.n_kv_heads = (int32_t)R;
  sel.head_dim = TKV_D;
  sel.n_channels = 16;
  sel.top_k = d->top_k;
  sel.n_sink = 0;
  sel.n_window = 1;
  sel.capacity = (int32_t)stride;
  sel.batch = 1;
  size_t off[6];
  const size_t sel_bytes = tkv::sparse_ws_layout(&sel, off, nullptr);
  size_t o = 0;
  const size_t o_sel = o;      o = tkv::align16(o + sel_bytes);  // first: its head must be zero-filled
  const size_t o_scores = o;   o = tkv::align16(o + R * stride * 4);
  const size_t o_ml = o;       o = tkv::align16(o + R * (size_t)ntb * 8);
  const size_t o_idx = o;      o = tkv::align16(o + R * (size_t)d->top_k * 4);
  const size_t o_cnt = o;      o = tkv::align16(o + R * 4);
  const size_t o_rowp = o;     o = tkv::align16(o + R * 4);
  if (out) {
    out->select_ws = base + o_sel;
    out->scores = (float*)(base + o_scores);
    out->ml = (float*)(base + o_ml);
    out->topk_idx = (int32_t*)(base + o_idx);
    out->topk_count = (int32_t*)(base + o_cnt);
    out->row_p = (float*)(base + o_rowp);
    out->stride = stride;
    out->ntb = ntb;
    out->sel = sel;
  }
  return o;
}

}  // namespace

extern "C" int32_t tkv_dense_preference_sizes(const tkv_pref_desc* d, size_t* workspace_bytes) {
  int32_t st = check_pref_desc(d);
  if (st != TKV_OK) return st;
  if (!workspace_bytes) return TKV_E_INVAL;
  *workspace_bytes = pref_ws_layout(d, nullptr, nullptr) + 256;
  return TKV_OK;
}

extern "C" int32_t tkv_dense_preference(const tkv_pref_desc* d, const void* q_last, const void* k, int32_t n,
                                        float sm_scale, float* p_out, void* workspace, size_t workspace_bytes,
                                        void* stream) {
  int32_t st = check_pref_desc(d);
  if (st != TKV_OK) return st;
  if (!q_last || !k || !p_out || !workspace || n < 1) return TKV_E_INVAL;
  if (n > d->capacity) return TKV_E_CAPACITY;
  if (workspace_bytes < pref_ws_layout(d, nullptr, nullptr)) return TKV_E_WORKSPACE;
  PrefWs ws;
  pref_ws_layout(d, (char*)workspace, &ws);
  const tkv::SparseWs sws = tkv::carve_sparse_ws(&ws.sel, ws.select_ws);
  const int G = d->n_q_heads / d->n_kv_heads, R = G * d->n_q;
  hipStream_t s = (hipStream_t)stream;
  PrefParams p;
  p.q_last = (const __half*)q_last;
  p.k = (const __half*)k;
  p.scores = ws.scores;
  p.ml = ws.ml;
  p.topk_idx = ws.topk_idx;
  p.topk_count = ws.topk_count;
  p.row_p = ws.row_p;
  p.p_out = p_out;
  p.scale2 = sm_scale * 1.44269504088896340736f;
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.n_q = d->n_q;
  p.n = n;
  p.ntb = (n + kTokBlock - 1) / kTokBlock;
  p.top_k = d->top_k;
  p.stride = ws.stride;
  // one (sequence, KV head) at a time: the logits of its G * n_q rows stay in the workspace
  for (int b = 0; b < d->batch; ++b) {
    for (int h = 0; h < d->n_kv_heads; ++h) {
      p.b = b;
      p.h = h;
      TKV_LAUNCH(pref_logits_kernel, dim3(p.ntb, (R / 16 + 3) / 4), 256, 0, s, p);
      st = tkv::topk_of_scores(ws.scores, ws.stride, R, n, d->top_k, (int)ws.stride, sws, ws.topk_idx, ws.topk_count, s);
      if (st != TKV_OK) return st;
      TKV_LAUNCH(pref_row_kernel, dim3(R), 256, 0, s, p);
      TKV_LAUNCH(pref_sum_kernel, 1, 64, 0, s, p);
    }
  }
  return TKV_OK;
}

extern "C" int32_t tkv_classify_layer(const float* p_heads_host, int32_t n_heads, int32_t n_q, float tau,
                                      float* layer_score_out) {
  if (!p_heads_host || n_heads <= 0 || n_q <= 0) return TKV_E_INVAL;
  double sum = 0.0;
  for (int i = 0; i < n_heads; ++i) sum += (double)p_heads_host[i];
  const double score = sum / n_heads / n_q;
  if (layer_score_out) *layer_score_out = (float)score;
  return score > (double)tau ? 1 : 0;
}
