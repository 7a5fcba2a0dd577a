// tkv_quant_attn_decode: Eq. 3 (Sec. 2.1) over the dequantized cache of a
// quantization-friendly layer (Sec. 4.3), split over token chunks with a
// log-sum-exp merge.
#include <atomic>
#include <mutex>

#include "tkv_common.h"

namespace tkv {
// matrix-core path (tkv_quant_attn_mfma.hip); returns TKV_E_UNSUPPORTED when the
// shape is not one it is built for.
int32_t launch_quant_attn_mfma(const tkv_quant_desc* d, const tkv_quant_cache* c, const __half* q, __half* out,
                               float scale2, float* parts, size_t parts_floats, uint32_t* arrivals, int target_blocks,
                               int max_groups, int max_tail, const TkvSeqLens& lens, const QuantNewTokens* fresh,
                               hipStream_t s);
}  // namespace tkv

namespace {

std::atomic<int> g_kernel_choice{0};      // 0: matrix-core kernel (+ reference kernel for the tail), 1: reference kernel only
std::atomic<int> g_target_blocks{0};      // workgroups the split-K launch aims at; 0 = one per compute unit of the stream

struct QuantAttnParams {
  const uint32_t* k_codes;
  const uint32_t* v_codes;
  const __half* k_scale;
  const __half* k_zero;
  const __half* v_scale;
  const __half* v_zero;
  const __half* k_resid;
  const __half* v_resid;
  const __half* q;
  float* parts;  // [B][Hq][n_chunks + 1][D + 4]
  float scale2;  // sm_scale * log2(e)
  int32_t hq, hkv, bits, group, residual, capacity;
  int32_t groups_per_chunk, n_chunks;  // chunk size in blocks of 32 tokens
  int32_t chunk_offset;  // blockIdx.x + chunk_offset is the chunk; chunk == n_chunks is the fp16 tail
  TkvSeqLens lens;
};

__device__ inline float wave_half_max(float v) {
  // max over the 32 lanes that share l / 32
  for (int m = 16; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

// Shape-generic reference kernel: plain float32 arithmetic, one wave per 32-token
// block, no matrix cores.  Correct for every supported descriptor; the tuned
// kernel takes over where it applies.
__global__ __launch_bounds__(256) void quant_attn_generic_kernel(QuantAttnParams p) {
  __shared__ float qs[4][TKV_D];            // query heads of this KV head, zero padded
  __shared__ float ksz[4][TKV_D][2];        // per wave: K scale, zero of the current group
  __shared__ float pw[4][4][TKV_BLK];       // per wave: weights p[h][t]
  __shared__ float alpha_s[4][4];           // per wave: rescale factors
  __shared__ uint32_t vblk[4][TKV_D * 4];   // per wave: packed V block (<= 512 words)
  __shared__ float red_m[4][4], red_l[4][4];
  __shared__ float red_o[4][4][TKV_D];

  // Groups of more than 4 query heads per KV head are served 4 heads at a time: blockIdx.y runs
  // over (KV head, quarter of its group).
  const int split = (p.hq / p.hkv + 3) / 4;
  const int b = blockIdx.z, h = blockIdx.y / split, chunk = blockIdx.x + p.chunk_offset;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int qh0 = h * (p.hq / p.hkv) + 4 * (blockIdx.y % split);  // first query head of this workgroup
  const int G = min(4, (h + 1) * (p.hq / p.hkv) - qh0);
  const int n = p.lens.n[b];
  const int nq = tkv::n_quantized(n, p.residual, p.group);
  const int jq = nq / TKV_BLK;  // packed blocks of 32 tokens
  const size_t bh = (size_t)b * p.hkv + h;
  const size_t n_blocks_cap = (size_t)(p.capacity / TKV_BLK);
  const size_t n_groups_cap = (size_t)(p.capacity / p.group);
  const int bpg = p.group / TKV_BLK;  // blocks per key group
  const int nu = TKV_D / p.group;     // channel groups of a value row
  const int nwords = TKV_D * p.bits;
  const int ring = p.residual + p.group;
  const bool tail = chunk == p.n_chunks;

  for (int i = tid; i < 4 * TKV_D; i += 256) {
    const int hh = i / TKV_D, c = i % TKV_D;
    qs[hh][c] = hh < G ? __half2float(p.q[((size_t)b * p.hq + (size_t)qh0 + hh) * TKV_D + c]) : 0.f;
  }
  __syncthreads();

  // blocks of 32 tokens this workgroup owns: [blk0, blk1)
  int blk0, blk1;
  if (!tail) {
    blk0 = chunk * p.groups_per_chunk;
    blk1 = min(blk0 + p.groups_per_chunk, jq);
  } else {
    blk0 = 0;
    blk1 = (n - nq + TKV_BLK - 1) / TKV_BLK;
  }

  const int t = lane % 32, hp = lane / 32;
  float m_run[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  float l_run[4] = {0.f, 0.f, 0.f, 0.f};
  float o_run[4][2] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};
  const int c0 = 2 * lane, u = c0 / p.group;

  for (int blk = blk0 + wave; blk < blk1; blk += 4) {
    float acc0 = 0.f, acc1 = 0.f;
    bool valid = true;
    if (!tail) {
      const size_t grp = bh * n_blocks_cap + blk;            // packed block
      const size_t kgrp = bh * n_groups_cap + blk / bpg;     // its key group
      // K scale / zero of this group -> LDS
      for (int c = lane; c < TKV_D; c += 64) {
        ksz[wave][c][0] = __half2float(p.k_scale[kgrp * TKV_D + c]);
        ksz[wave][c][1] = __half2float(p.k_zero[kgrp * TKV_D + c]);
      }
      for (int w = lane; w < nwords; w += 64) vblk[wave][w] = p.v_codes[grp * nwords + w];
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_s_waitcnt(0);
      const uint32_t* kblk = p.k_codes + grp * nwords;
      const uint32_t cmask = (1u << p.bits) - 1u;
      for (int c = 0; c < TKV_D; ++c) {
        int w, f;
        tkv::k_code_pos(p.bits, t, c, w, f);
        const float code = (float)((kblk[w] >> (p.bits * f)) & cmask);
        const float kh = code * ksz[wave][c][0] + ksz[wave][c][1];
        acc0 += qs[2 * hp][c] * kh;
        acc1 += qs[2 * hp + 1][c] * kh;
      }
    } else {
      const int tok = nq + blk * TKV_BLK + t;
      valid = tok < n;
      if (valid) {
        const __half* krow = p.k_resid + (bh * ring + (size_t)(tok % ring)) * TKV_D;
        for (int c = 0; c < TKV_D; ++c) {
          const float kh = __half2float(krow[c]);
          acc0 += qs[2 * hp][c] * kh;
          acc1 += qs[2 * hp + 1][c] * kh;
        }
      }
    }
    const float x0 = valid ? acc0 * p.scale2 : -INFINITY;
    const float x1 = valid ? acc1 * p.scale2 : -INFINITY;
    const float g0 = wave_half_max(x0), g1 = wave_half_max(x1);
    // publish p and alpha for this wave
    {
      const float mo0 = m_run[2 * hp], mo1 = m_run[2 * hp + 1];
      const float mn0 = fmaxf(mo0, g0), mn1 = fmaxf(mo1, g1);
      pw[wave][2 * hp][t] = exp2f(x0 - mn0);
      pw[wave][2 * hp + 1][t] = exp2f(x1 - mn1);
      if (t == 0) {
        alpha_s[wave][2 * hp] = exp2f(mo0 - mn0);
        alpha_s[wave][2 * hp + 1] = exp2f(mo1 - mn1);
      }
      // every lane tracks all four maxima; fetch the other half's via LDS below
      red_m[wave][2 * hp] = mn0;
      red_m[wave][2 * hp + 1] = mn1;
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0);
    float al[4];
    for (int hh = 0; hh < 4; ++hh) {
      al[hh] = alpha_s[wave][hh];
      m_run[hh] = red_m[wave][hh];
    }
    // P.V for channels c0, c0+1
    float s0[4] = {0.f, 0.f, 0.f, 0.f}, s1[4] = {0.f, 0.f, 0.f, 0.f}, ls[4] = {0.f, 0.f, 0.f, 0.f};
    for (int tt = 0; tt < TKV_BLK; ++tt) {
      float v0, v1;
      if (!tail) {
        const size_t grp = bh * n_blocks_cap + blk;
        const float sc = __half2float(p.v_scale[(grp * nu + u) * TKV_BLK + tt]);
        const float ze = __half2float(p.v_zero[(grp * nu + u) * TKV_BLK + tt]);
        const uint32_t cmask = (1u << p.bits) - 1u;
        int w, f;
        tkv::v_code_pos(p.bits, tt, c0, w, f);
        v0 = (float)((vblk[wave][w] >> (p.bits * f)) & cmask) * sc + ze;
        tkv::v_code_pos(p.bits, tt, c0 + 1, w, f);
        v1 = (float)((vblk[wave][w] >> (p.bits * f)) & cmask) * sc + ze;
      } else {
        const int tok = nq + blk * TKV_BLK + tt;
        if (tok < n) {
          const __half* vrow = p.v_resid + (bh * ring + (size_t)(tok % ring)) * TKV_D;
          v0 = __half2float(vrow[c0]);
          v1 = __half2float(vrow[c0 + 1]);
        } else {
          v0 = v1 = 0.f;
        }
      }
      for (int hh = 0; hh < 4; ++hh) {
        const float pp = pw[wave][hh][tt];
        s0[hh] += pp * v0;
        s1[hh] += pp * v1;
        ls[hh] += pp;
      }
    }
    for (int hh = 0; hh < 4; ++hh) {
      o_run[hh][0] = o_run[hh][0] * al[hh] + s0[hh];
      o_run[hh][1] = o_run[hh][1] * al[hh] + s1[hh];
      l_run[hh] = l_run[hh] * al[hh] + ls[hh];
    }
    __builtin_amdgcn_wave_barrier();
  }

  // merge the four waves
  __syncthreads();
  if (lane == 0)
    for (int hh = 0; hh < 4; ++hh) {
      red_m[wave][hh] = m_run[hh];
      red_l[wave][hh] = l_run[hh];
    }
  for (int hh = 0; hh < 4; ++hh) {
    red_o[wave][hh][c0] = o_run[hh][0];
    red_o[wave][hh][c0 + 1] = o_run[hh][1];
  }
  __syncthreads();
  const int n_parts = p.n_chunks + 1;
  for (int i = tid; i < G * TKV_D; i += 256) {
    const int hh = i / TKV_D, c = i % TKV_D;
    float M = -INFINITY;
    for (int w = 0; w < 4; ++w) M = fmaxf(M, red_m[w][hh]);
    float L = 0.f, O = 0.f;
    for (int w = 0; w < 4; ++w) {
      const float mw = red_m[w][hh];
      const float wgt = mw == -INFINITY ? 0.f : exp2f(mw - M);
      L += red_l[w][hh] * wgt;
      O += red_o[w][hh][c] * wgt;
    }
    float* dst = p.parts + (((size_t)b * p.hq + (size_t)qh0 + hh) * n_parts + chunk) * TKV_PART_STRIDE;
    dst[TKV_PART_O + c] = O;
    if (c == 0) {
      dst[0] = M;
      dst[1] = L;
    }
  }
}

// Log-sum-exp merge of the chunk partials of one query head; writes fp16.
// One workgroup per query head, one thread per channel; the per-part maxima and sums
// are staged in LDS so that the channel loop issues independent loads.
__global__ __launch_bounds__(TKV_D) void attn_merge_kernel(const float* parts, __half* out, int n_parts) {
  __shared__ float wgt[TKV_MAX_CHUNKS + 1];
  __shared__ float red[2];
  const size_t head = blockIdx.x;  // b * Hq + i
  const int c = threadIdx.x;
  const float* base = parts + head * n_parts * TKV_PART_STRIDE;
  for (int k = c; k < n_parts; k += TKV_D) wgt[k] = base[(size_t)k * TKV_PART_STRIDE];
  __syncthreads();
  float M = -INFINITY;
  for (int k = 0; k < n_parts; ++k) M = fmaxf(M, wgt[k]);
  __syncthreads();
  float lsum = 0.f;
  for (int k = c; k < n_parts; k += TKV_D) {
    const float mk = wgt[k];
    const float w = mk == -INFINITY ? 0.f : exp2f(mk - M);
    wgt[k] = w;
    lsum += w * base[(size_t)k * TKV_PART_STRIDE + 1];
  }
  for (int m = 32; m >= 1; m >>= 1) lsum += __shfl_xor(lsum, m, 64);
  if (c % 64 == 0) red[c / 64] = lsum;
  __syncthreads();
  const float L = red[0] + red[1];
  float O0 = 0.f, O1 = 0.f, O2 = 0.f, O3 = 0.f;
  int k = 0;
  for (; k + 4 <= n_parts; k += 4) {
    const float* pk = base + (size_t)k * TKV_PART_STRIDE + TKV_PART_O + c;
    const float v0 = pk[0], v1 = pk[TKV_PART_STRIDE], v2 = pk[2 * TKV_PART_STRIDE], v3 = pk[3 * TKV_PART_STRIDE];
    O0 = __builtin_fmaf(v0, wgt[k], O0);
    O1 = __builtin_fmaf(v1, wgt[k + 1], O1);
    O2 = __builtin_fmaf(v2, wgt[k + 2], O2);
    O3 = __builtin_fmaf(v3, wgt[k + 3], O3);
  }
  for (; k < n_parts; ++k) O0 = __builtin_fmaf(base[(size_t)k * TKV_PART_STRIDE + TKV_PART_O + c], wgt[k], O0);
  const float O = (O0 + O1) + (O2 + O3);
  out[head * TKV_D + c] = __float2half_rn(L > 0.f ? O / L : 0.f);
}

}  // namespace

namespace tkv {
int32_t launch_attn_merge(const float* parts, __half* out, int n_heads_total, int n_parts, hipStream_t s) {
  TKV_LAUNCH(attn_merge_kernel, dim3(n_heads_total), TKV_D, 0, s, parts, out, n_parts);
  return TKV_OK;
}
}  // namespace tkv

extern "C" int32_t tkv_debug_quant_attn_config(int32_t kernel_choice, int32_t target_blocks) {
  if (kernel_choice < 0 || kernel_choice > 1 || target_blocks < -1) return TKV_E_INVAL;
  g_kernel_choice = kernel_choice;
  if (target_blocks > 0) g_target_blocks = target_blocks;
  if (target_blocks == -1) g_target_blocks = 0;  // back to one workgroup per compute unit of the stream
  return TKV_OK;
}

namespace {

// Body of both entry points.  parts: room for parts_floats floats of split-K partials; arrivals:
// one zero word per (sequence, KV head, four query heads of its group).  TKV_E_WORKSPACE if the launch's partials do not fit.
// fresh: the step's new tokens, already counted in seq_len_host but not yet in the fp16 ring (the
// matrix-core kernel reads them from the caller's buffers and writes them into the ring); only
// with the matrix-core kernel (TKV_E_UNSUPPORTED otherwise, before anything is launched).
int32_t quant_attn_decode_impl(const tkv_quant_desc* d, const tkv_quant_cache* c, const void* q, void* out,
                               float sm_scale, float* parts, size_t parts_floats, uint32_t* arrivals,
                               hipStream_t s, const tkv::QuantNewTokens* fresh = nullptr) {
  QuantAttnParams p;
  int max_groups = 0, max_tail = 0;
  for (int b = 0; b < d->batch; ++b) {
    const int32_t n = c->seq_len_host[b];
    if (n < 0) return TKV_E_INVAL;
    if (n > d->capacity) return TKV_E_CAPACITY;
    p.lens.n[b] = n;
    const int g = tkv::n_quantized(n, d->residual, d->group_size) / TKV_BLK;  // in blocks of 32 tokens
    if (g > max_groups) max_groups = g;
    if (n - g * TKV_BLK > max_tail) max_tail = n - g * TKV_BLK;
  }
  // Chunking of the reference kernel: about 1024 workgroups over the whole launch.
  const int bh = d->batch * d->n_kv_heads;
  int target = (1024 + bh - 1) / bh;
  if (target > TKV_MAX_CHUNKS) target = TKV_MAX_CHUNKS;
  if (target < 1) target = 1;
  int gpc = (max_groups + target - 1) / target;
  if (gpc < 4) gpc = 4;
  int n_chunks = (max_groups + gpc - 1) / gpc;
  if (n_chunks < 1) n_chunks = 1;

  p.k_codes = (const uint32_t*)c->k_codes;
  p.v_codes = (const uint32_t*)c->v_codes;
  p.k_scale = (const __half*)c->k_scale;
  p.k_zero = (const __half*)c->k_zero;
  p.v_scale = (const __half*)c->v_scale;
  p.v_zero = (const __half*)c->v_zero;
  p.k_resid = (const __half*)c->k_resid;
  p.v_resid = (const __half*)c->v_resid;
  p.q = (const __half*)q;
  p.parts = parts;
  p.scale2 = sm_scale * 1.44269504088896340736f;
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.bits = d->bits;
  p.group = d->group_size;
  p.residual = d->residual;
  p.capacity = d->capacity;
  p.groups_per_chunk = gpc;
  p.n_chunks = n_chunks;

  if (g_kernel_choice.load() == 0) {
    // matrix-core kernel: one launch covers the quantized groups and the fp16 tail
    int target_blocks = g_target_blocks.load();
    // one workgroup per compute unit that the stream may use: on a stream with a compute-unit
    // mask a launch sized for the whole machine would leave a few workgroups for a second round
    if (target_blocks == 0) target_blocks = tkv::stream_compute_units(s);
    const int32_t st = tkv::launch_quant_attn_mfma(d, c, p.q, (__half*)out, p.scale2, p.parts, parts_floats, arrivals,
                                                   target_blocks, max_groups, max_tail, p.lens, fresh, s);
    if (st != TKV_E_UNSUPPORTED) return st;
  }
  if (fresh != nullptr) return TKV_E_UNSUPPORTED;
  // reference kernel: on request, and for the settings the matrix-core kernel is not built for
  if ((size_t)d->batch * d->n_q_heads * (n_chunks + 1) * TKV_PART_STRIDE > parts_floats) return TKV_E_WORKSPACE;
  p.chunk_offset = 0;
  const int split = (d->n_q_heads / d->n_kv_heads + 3) / 4;
  TKV_LAUNCH(quant_attn_generic_kernel, dim3(n_chunks + 1, d->n_kv_heads * split, d->batch), 256, 0, s, p);
  return tkv::launch_attn_merge(p.parts, (__half*)out, d->batch * d->n_q_heads, n_chunks + 1, s);
}

int32_t check_decode_args(const tkv_quant_desc* d, const tkv_quant_cache* c, const void* q, const void* out) {
  const int32_t st = tkv::check_quant_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || !q || !out) return TKV_E_INVAL;
  if (!c->k_codes || !c->k_scale || !c->k_zero || !c->v_codes || !c->v_scale || !c->v_zero || !c->k_resid ||
      !c->v_resid)
    return TKV_E_INVAL;
  return TKV_OK;
}

}  // namespace

extern "C" int32_t tkv_quant_attn_decode(const tkv_quant_desc* d, const tkv_quant_cache* c, const void* q,
                                         void* out, float sm_scale, void* workspace, size_t workspace_bytes,
                                         void* stream) {
  int32_t st = check_decode_args(d, c, q, out);
  if (st != TKV_OK) return st;
  if (!workspace) return TKV_E_INVAL;
  size_t need = 0;
  tkv_quant_cache_sizes(d, nullptr, &need);
  if (workspace_bytes < need) return TKV_E_WORKSPACE;
  // arrival counters sit behind the partials (zero before first use, left zero by every call)
  const size_t parts_floats = (size_t)d->batch * d->n_q_heads * (TKV_MAX_CHUNKS + 1) * TKV_PART_STRIDE;
  uint32_t* arrivals = (uint32_t*)((char*)workspace + ((parts_floats * sizeof(float) + 255) & ~(size_t)255));
  return quant_attn_decode_impl(d, c, q, out, sm_scale, (float*)workspace, parts_floats, arrivals, (hipStream_t)stream);
}

// ---- tkv_quant_decode: Eq. 2 and Eq. 3 of a quantized layer's decode step in one call ----------
extern "C" int32_t tkv_quant_decode(const tkv_quant_desc* d, tkv_quant_cache* c, const void* k_new,
                                    const void* v_new, int32_t n_new, const int32_t* n_valid_host, const void* q,
                                    void* out, float sm_scale, void* workspace, size_t workspace_bytes,
                                    void* stream) {
  int32_t st = check_decode_args(d, c, q, out);
  if (st != TKV_OK) return st;
  if (!workspace || n_new < 0 || (n_new > 0 && (!k_new || !v_new))) return TKV_E_INVAL;
  size_t need = 0;
  tkv_quant_cache_sizes(d, nullptr, &need);
  if (workspace_bytes < need) return TKV_E_WORKSPACE;
  if (n_new == 0) return tkv_quant_attn_decode(d, c, q, out, sm_scale, workspace, workspace_bytes, stream);
  // One launch when no sequence completes a quantization group with these tokens (the new rows
  // then only join the fp16 ring, which the attention kernel does itself) and the matrix-core
  // kernel serves the descriptor; else the append's launches, then the attention's.
  tkv::QuantNewTokens fresh;
  fresh.k_new = (const __half*)k_new;
  fresh.v_new = (const __half*)v_new;
  fresh.n_stride = n_new;
  bool one_launch = g_kernel_choice.load() == 0 && d->head_dim == TKV_D;
  {
    const int variant = d->bits * 100 + d->group_size;
    if (variant != 232 && variant != 432 && variant != 164 && variant != 264) one_launch = false;
  }
  for (int b = 0; b < d->batch; ++b) {
    const int64_t n0 = c->seq_len_host[b];
    const int32_t add = n_valid_host ? n_valid_host[b] : n_new;
    if (n0 < 0 || add < 0 || add > n_new) return TKV_E_INVAL;
    if (n0 + add > d->capacity) return TKV_E_CAPACITY;
    fresh.n_add.n[b] = add;
    const int32_t g = d->group_size;
    if (tkv::n_quantized((int32_t)n0 + add, d->residual, g) != tkv::n_quantized((int32_t)n0, d->residual, g))
      one_launch = false;
  }
  if (!one_launch) {
    st = tkv_quantize_append_ragged(d, c, k_new, v_new, n_new, n_valid_host, stream);
    if (st != TKV_OK) return st;
    return tkv_quant_attn_decode(d, c, q, out, sm_scale, workspace, workspace_bytes, stream);
  }
  const size_t parts_floats = (size_t)d->batch * d->n_q_heads * (TKV_MAX_CHUNKS + 1) * TKV_PART_STRIDE;
  uint32_t* arrivals = (uint32_t*)((char*)workspace + ((parts_floats * sizeof(float) + 255) & ~(size_t)255));
  for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] += fresh.n_add.n[b];
  st = quant_attn_decode_impl(d, c, q, out, sm_scale, (float*)workspace, parts_floats, arrivals, (hipStream_t)stream,
                              &fresh);
  if (st != TKV_OK)  // nothing was launched: the cache is as it was
    for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] -= fresh.n_add.n[b];
  return st;
}

// ---- tkv_quant_attn_decode for callers that cannot hand over a workspace -----------------
// The split-K partials and arrival counters live in a fixed array in device memory that is part
// of the library image (every GPU the library runs on holds its own copy until the process
// ends).  In host code the array's name is only a stand-in for the symbol: the address that
// kernels may use is looked up once per device with that device current.
namespace {

constexpr size_t kStaticCounterWords = TKV_STATIC_MAX_HEADS;   // one per (sequence, KV head, four query heads)
constexpr size_t kStaticPartsBytes = TKV_STATIC_PARTS_BYTES;
constexpr size_t kStaticBytes = kStaticCounterWords * sizeof(uint32_t) + kStaticPartsBytes;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_static_ptr[kMaxDevices] = {};  // device address of `scratch` on each device

int32_t static_scratch(unsigned char** ptr_out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TKV_E_HIP;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return TKV_E_HIP;
    g_static_ptr[dev] = (unsigned char*)ptr;
  }
  *ptr_out = g_static_ptr[dev];
  return TKV_OK;
}

// Clears the arrival counters (a fill kernel, not a memset node: the call may be recorded
// into a graph by its caller).
__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t* dst, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = 0u;
}

}  // namespace

extern "C" int32_t tkv_quant_attn_decode_static(const tkv_quant_desc* d, const tkv_quant_cache* c, const void* q,
                                                void* out, float sm_scale, void* stream) {
  int32_t st = check_decode_args(d, c, q, out);
  if (st != TKV_OK) return st;
  const int bh = d->batch * d->n_kv_heads * ((d->n_q_heads / d->n_kv_heads + 3) / 4);
  if ((size_t)bh > kStaticCounterWords) return TKV_E_WORKSPACE;
  unsigned char* base = nullptr;
  st = static_scratch(&base);
  if (st != TKV_OK) return st;
  uint32_t* arrivals = (uint32_t*)base;
  float* parts = (float*)(base + kStaticCounterWords * sizeof(uint32_t));
  hipStream_t s = (hipStream_t)stream;
  // the array keeps whatever the previous call left: the counters must start at zero
  TKV_LAUNCH(clear_words_kernel, dim3((bh + 255) / 256), 256, 0, s, arrivals, bh);
  return quant_attn_decode_impl(d, c, q, out, sm_scale, parts, kStaticPartsBytes / sizeof(float), arrivals, s);
}
