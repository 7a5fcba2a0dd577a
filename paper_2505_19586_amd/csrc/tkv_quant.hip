// tkv_quantize_append: cache update (Sec. 2.1, Eq. 2) and static quantization of the
// groups that become complete (Sec. 2.2, Eq. 4; Sec. 4.3: keys per channel, values
// per token; fp16 zero-point and scaler, Sec. 4.4).
#include "tkv_common.h"

// The quantizer's float32 operations are part of the contract (each a single
// rounded operation); keep the compiler from fusing any of them.
#pragma clang fp contract(off)

namespace {

struct QuantAppendParams {
  uint32_t* k_codes;
  uint32_t* v_codes;
  __half* k_scale;
  __half* k_zero;
  __half* v_scale;
  __half* v_zero;
  __half* k_resid;
  __half* v_resid;
  const __half* k_new;
  const __half* v_new;
  int32_t hkv, bits, group, residual, capacity;
  int32_t n_stride;   // rows per sequence in k_new / v_new
  TkvSeqLens n_old;
  TkvSeqLens n_add;   // valid new rows per sequence (<= n_stride)
};

__device__ inline float quant_code(float x, float z, float s, float qmax) {
  // Eq. 4 with the stored fp16 s and z; one subtraction, one division, rint.
  const float d = x - z;
  const float t = d / s;
  float c = rintf(t);
  c = fminf(fmaxf(c, 0.0f), qmax);
  return s == 0.0f ? 0.0f : c;
}

// One workgroup quantizes one group of GRP tokens of one KV head.  BITS and GRP are template
// parameters so that the packed-layout index arithmetic folds to shifts and masks.
template <int BITS, int GRP>
__global__ __launch_bounds__(256) void quantize_group_kernel(QuantAppendParams p) {
  constexpr int NU = TKV_D / GRP;     // channel groups of a value row
  constexpr int NB = GRP / TKV_BLK;   // code blocks of a token group
  __shared__ __half kt[GRP][TKV_D];
  __shared__ __half vt[GRP][TKV_D];
  __shared__ float ks[TKV_D], kz[TKV_D];
  __shared__ float vs[GRP][NU], vz[GRP][NU];

  const int b = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const int n0 = p.n_old.n[b], n1 = n0 + p.n_add.n[b];
  const int j0 = tkv::n_quantized(n0, p.residual, GRP) / GRP;
  const int j1 = tkv::n_quantized(n1, p.residual, GRP) / GRP;
  const int j = j0 + (int)blockIdx.x;
  if (j >= j1) return;
  const int ring = p.residual + GRP;
  const size_t bh = (size_t)b * p.hkv + h;
  const size_t n_groups_cap = (size_t)(p.capacity / GRP);
  const size_t n_blocks_cap = (size_t)(p.capacity / TKV_BLK);

  // stage the group's K rows and V rows (16-byte chunks)
  for (int i = tid; i < GRP * 16; i += 256) {
    const int t = i / 16, part = i % 16;
    const int tok = GRP * j + t;
    const uint4 *ksrc, *vsrc;
    if (tok < n0) {
      const size_t row = (bh * ring + (size_t)(tok % ring)) * TKV_D;
      ksrc = reinterpret_cast<const uint4*>(p.k_resid + row);
      vsrc = reinterpret_cast<const uint4*>(p.v_resid + row);
    } else {
      const size_t row = (((size_t)b * p.n_stride + (size_t)(tok - n0)) * p.hkv + h) * TKV_D;
      ksrc = reinterpret_cast<const uint4*>(p.k_new + row);
      vsrc = reinterpret_cast<const uint4*>(p.v_new + row);
    }
    reinterpret_cast<uint4*>(&kt[t][0])[part] = ksrc[part];
    reinterpret_cast<uint4*>(&vt[t][0])[part] = vsrc[part];
  }
  __syncthreads();

  constexpr float qmax = (float)((1 << BITS) - 1);
  if (tid < TKV_D) {
    // keys: one (s, z) per channel over the group's tokens
    const int c = tid;
    float mn = __half2float(kt[0][c]), mx = mn;
    for (int t = 1; t < GRP; ++t) {
      const float x = __half2float(kt[t][c]);
      mn = fminf(mn, x);
      mx = fmaxf(mx, x);
    }
    const float range = mx - mn;
    const float s32 = range / qmax;
    const __half s16 = __float2half_rn(s32);
    const __half z16 = __float2half_rn(mn);  // exact: mn is an fp16 value
    const size_t o = (bh * n_groups_cap + j) * TKV_D + c;
    p.k_scale[o] = s16;
    p.k_zero[o] = z16;
    ks[c] = __half2float(s16);
    kz[c] = __half2float(z16);
  } else {
    // values: one (s, z) per token and channel group; 128 threads cover GRP * NU = 128 pairs
    const int pr = tid - TKV_D;
    const int t = pr / NU, u = pr % NU;
    float mn = 0.f, mx = 0.f;
    for (int i = 0; i < GRP; ++i) {
      const int c = GRP * u + ((i + pr) % GRP);  // rotated start: fewer LDS bank conflicts
      const float x = __half2float(vt[t][c]);
      mn = i == 0 ? x : fminf(mn, x);
      mx = i == 0 ? x : fmaxf(mx, x);
    }
    const float range = mx - mn;
    const float s32 = range / qmax;
    const __half s16 = __float2half_rn(s32);
    const __half z16 = __float2half_rn(mn);
    // stored per block of 32 tokens as [u][t]
    const size_t blk = (size_t)j * NB + t / TKV_BLK;
    const size_t o = ((bh * n_blocks_cap + blk) * NU + u) * TKV_BLK + t % TKV_BLK;
    p.v_scale[o] = s16;
    p.v_zero[o] = z16;
    vs[t][u] = __half2float(s16);
    vz[t][u] = __half2float(z16);
  }
  __syncthreads();

  constexpr int nwords = TKV_D * BITS;  // words of one packed block: 32*128*bits/32
  constexpr int nfields = 32 / BITS;
  uint32_t* kdst = p.k_codes + (bh * n_blocks_cap + (size_t)j * NB) * (size_t)nwords;
  uint32_t* vdst = p.v_codes + (bh * n_blocks_cap + (size_t)j * NB) * (size_t)nwords;
#pragma unroll
  for (int w0 = 0; w0 < NB * nwords; w0 += 256) {
    const int wi = w0 + tid;
    if ((NB * nwords) % 256 != 0 && wi >= NB * nwords) break;
    const int blk = wi / nwords, w = wi % nwords;  // block of the group, word of the block
    uint32_t kw = 0, vw = 0;
#pragma unroll
    for (int f = 0; f < nfields; ++f) {
      int t, c;
      tkv::k_code_elem(BITS, w, f, t, c);
      t += TKV_BLK * blk;
      const float kc = quant_code(__half2float(kt[t][c]), kz[c], ks[c], qmax);
      kw |= (uint32_t)kc << (BITS * f);
      tkv::v_code_elem(BITS, w, f, t, c);
      t += TKV_BLK * blk;
      const float vc = quant_code(__half2float(vt[t][c]), vz[t][c / GRP], vs[t][c / GRP], qmax);
      vw |= (uint32_t)vc << (BITS * f);
    }
    kdst[wi] = kw;
    vdst[wi] = vw;
  }
}

// Copies the new tokens that stay unquantized into the fp16 ring.  Runs after
// quantize_group_kernel so that ring slots of tokens just quantized may be reused.
__global__ __launch_bounds__(256) void ring_update_kernel(QuantAppendParams p) {
  const int b = blockIdx.y, tid = threadIdx.x;
  const int n0 = p.n_old.n[b], n1 = n0 + p.n_add.n[b];
  const int nq1 = tkv::n_quantized(n1, p.residual, p.group);
  const int tok = n1 - 1 - (int)blockIdx.x;
  const int first = n0 > nq1 ? n0 : nq1;
  if (tok < first) return;
  const int ring = p.residual + p.group;
  const int chunks = p.hkv * 16;  // 16-byte chunks per token, K or V
  for (int i = tid; i < 2 * chunks; i += 256) {
    const int kv = i / chunks, rem = i % chunks;
    const int h = rem / 16, part = rem % 16;
    const __half* src = (kv ? p.v_new : p.k_new) + (((size_t)b * p.n_stride + (size_t)(tok - n0)) * p.hkv + h) * TKV_D;
    __half* dst = (kv ? p.v_resid : p.k_resid) + (((size_t)b * p.hkv + h) * ring + (size_t)(tok % ring)) * TKV_D;
    reinterpret_cast<uint4*>(dst)[part] = reinterpret_cast<const uint4*>(src)[part];
  }
}

}  // namespace

extern "C" int32_t tkv_quantize_append_ragged(const tkv_quant_desc* d, tkv_quant_cache* c, const void* k_new,
                                              const void* v_new, int32_t n_new, const int32_t* n_valid_host,
                                              void* stream) {
  int32_t st = tkv::check_quant_desc(d);
  if (st != TKV_OK) return st;
  if (!c || !c->seq_len_host || n_new < 0) return TKV_E_INVAL;
  if (n_new == 0) return TKV_OK;
  if (!k_new || !v_new || !c->k_codes || !c->k_scale || !c->k_zero || !c->v_codes || !c->v_scale ||
      !c->v_zero || !c->k_resid || !c->v_resid)
    return TKV_E_INVAL;

  QuantAppendParams p;
  int max_groups = 0, max_copy = 0;
  for (int b = 0; b < d->batch; ++b) {
    const int64_t n0 = c->seq_len_host[b];
    const int32_t add = n_valid_host ? n_valid_host[b] : n_new;
    if (n0 < 0 || add < 0 || add > n_new) return TKV_E_INVAL;
    if (n0 + add > d->capacity) return TKV_E_CAPACITY;
    p.n_old.n[b] = (int32_t)n0;
    p.n_add.n[b] = add;
    const int32_t n1 = (int32_t)n0 + add;
    const int32_t g = d->group_size;
    const int groups = (tkv::n_quantized(n1, d->residual, g) - tkv::n_quantized((int32_t)n0, d->residual, g)) / g;
    const int32_t nq1 = tkv::n_quantized(n1, d->residual, g);
    const int copy = n1 - (n0 > nq1 ? (int32_t)n0 : nq1);
    if (groups > max_groups) max_groups = groups;
    if (copy > max_copy) max_copy = copy;
  }
  p.k_codes = (uint32_t*)c->k_codes;
  p.v_codes = (uint32_t*)c->v_codes;
  p.k_scale = (__half*)c->k_scale;
  p.k_zero = (__half*)c->k_zero;
  p.v_scale = (__half*)c->v_scale;
  p.v_zero = (__half*)c->v_zero;
  p.k_resid = (__half*)c->k_resid;
  p.v_resid = (__half*)c->v_resid;
  p.k_new = (const __half*)k_new;
  p.v_new = (const __half*)v_new;
  p.hkv = d->n_kv_heads;
  p.bits = d->bits;
  p.group = d->group_size;
  p.residual = d->residual;
  p.capacity = d->capacity;
  p.n_stride = n_new;

  hipStream_t s = (hipStream_t)stream;
  if (max_groups > 0) {
    const dim3 grid(max_groups, d->n_kv_heads, d->batch);
    const int variant = d->bits * 100 + d->group_size;
    switch (variant) {
      case 132: TKV_LAUNCH((quantize_group_kernel<1, 32>), grid, 256, 0, s, p); break;
      case 232: TKV_LAUNCH((quantize_group_kernel<2, 32>), grid, 256, 0, s, p); break;
      case 432: TKV_LAUNCH((quantize_group_kernel<4, 32>), grid, 256, 0, s, p); break;
      case 164: TKV_LAUNCH((quantize_group_kernel<1, 64>), grid, 256, 0, s, p); break;
      case 264: TKV_LAUNCH((quantize_group_kernel<2, 64>), grid, 256, 0, s, p); break;
      case 464: TKV_LAUNCH((quantize_group_kernel<4, 64>), grid, 256, 0, s, p); break;
      default: return TKV_E_UNSUPPORTED;
    }
  }
  if (max_copy > 0) {
    TKV_LAUNCH(ring_update_kernel, dim3(max_copy, d->batch), 256, 0, s, p);
  }
  for (int b = 0; b < d->batch; ++b) c->seq_len_host[b] += p.n_add.n[b];
  return TKV_OK;
}

extern "C" int32_t tkv_quantize_append(const tkv_quant_desc* d, tkv_quant_cache* c, const void* k_new,
                                       const void* v_new, int32_t n_new, void* stream) {
  return tkv_quantize_append_ragged(d, c, k_new, v_new, n_new, nullptr, stream);
}
