// Matrix-core kernel of tkv_quant_attn_decode (Sec. 2.1 Eq. 3 over the quantized cache
// of Sec. 4.3) for gfx950, G = Hq/Hkv <= 4, D = 128, g = 32, bits 2 or 4.
//
// One wave64 owns one 32-token group at a time.  Both contractions run on
// v_mfma_f32_16x16x32_f16 with the packed codes as the A operand:
//
//   * a b-bit code c sitting at mantissa bits [bp, bp+b) of an otherwise zero fp16 IS
//     the subnormal number c * 2^bp * 2^-24, so one v_and_b32 per register turns two
//     codes into two exact fp16 operands (no bias, no convert); the 2^bp factor is
//     compensated in the other operand;
//   * q.K-hat = sum_c code[t][c] * (q[c] s[c]) + sum_c q[c] z[c]: the scaler moves into
//     the query operand (split into fp16 hi + lo parts so the product keeps ~22 bits),
//     the zero-point term is a second tiny MFMA per group;
//   * p.V-hat = sum_t code[t][d] * (p[t] s_v[t][u]) + sum_t p[t] z_v[t][u]: the 16
//     operand columns are the 4 query heads x 4 channel groups u, so the weights never
//     leave the lanes that produced them (the D layout of the first product is the B
//     layout of the second); z_v and the softmax denominator ride on one more MFMA.
//
// Softmax is online per wave with lazy rescaling; the four waves of a workgroup and the
// chunks of a sequence are merged with log-sum-exp merges.
#include <cstdlib>

#include "tkv_common.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

struct MfmaParams {
  const uint32_t* k_codes;
  const uint32_t* v_codes;
  const __half* k_scale;
  const __half* k_zero;
  const __half* v_scale;
  const __half* v_zero;
  const __half* k_resid;
  const __half* v_resid;
  const __half* q;
  float* parts;  // [B][Hq][n_chunks][D + 2]
  uint32_t* arrivals;  // [B][Hkv], zero between calls
  __half* out;         // [B][Hq][D]
  float scale2;
  int32_t hq, hkv, residual, capacity;
  int32_t n_chunks;
  int32_t dbg_mode;
  long long* dbg_ts;
  TkvSeqLens lens;
};

__device__ inline floatx4 mfma(uintx4 a, uintx4 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// Reinterpret one 32-bit register as two fp16.  Takes the word BY VALUE: applying
// __builtin_bit_cast directly to an element of an ext-vector (vec[j]) reads element 0
// for every j with this compiler.
__device__ inline half2_t as_half2(uint32_t w) { return __builtin_bit_cast(half2_t, w); }

__device__ inline uint32_t pack2(_Float16 lo, _Float16 hi) {
  half2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, v);
}

// fp16 hi/lo split of a product, written so that each part is one fused multiply-add
// with an fp16 result (the compiler selects v_fma_mixlo/mixhi_f16 for this shape):
//   hi = f16(a * b), lo = f16(a * b - hi)   (the FMA makes the residual exact)
// s2 holds two fp16 scalers; the results are packed the same way.  No inline assembly:
// the operands come straight from MFMA / transcendental results, whose read hazards
// only the compiler's own instructions are checked for.
__device__ inline uint32_t mix_hi_pair(float a0, float a1, uint32_t s2) {
  const half2_t s = as_half2(s2);
  return pack2((_Float16)__builtin_fmaf(a0, (float)s[0], 0.0f), (_Float16)__builtin_fmaf(a1, (float)s[1], 0.0f));
}
__device__ inline uint32_t mix_lo_pair(float a0, float a1, uint32_t s2, uint32_t hi) {
  const half2_t s = as_half2(s2), h = as_half2(hi);
  return pack2((_Float16)__builtin_fmaf(a0, (float)s[0], -(float)h[0]),
               (_Float16)__builtin_fmaf(a1, (float)s[1], -(float)h[1]));
}
// residual of rounding two floats to the packed fp16 pair `hi`: f16(a - hi)
__device__ inline uint32_t residual_pair(float a0, float a1, uint32_t hi) {
  const half2_t h = as_half2(hi);
  return pack2((_Float16)__builtin_fmaf(a0, 1.0f, -(float)h[0]), (_Float16)__builtin_fmaf(a1, 1.0f, -(float)h[1]));
}

// Two MFMA operands (8 registers) out of one 32-bit word of packed codes.
template <int BITS>
__device__ inline void extract(uint32_t w, uintx4& a0, uintx4& a1) {
  if (BITS == 2) {
    const uint32_t w8 = w >> 8;
    a0[0] = w & 0x00030003u;
    a0[1] = w & 0x000C000Cu;
    a0[2] = w & 0x00300030u;
    a0[3] = w & 0x00C000C0u;
    a1[0] = w8 & 0x00030003u;
    a1[1] = w8 & 0x000C000Cu;
    a1[2] = w8 & 0x00300030u;
    a1[3] = w8 & 0x00C000C0u;
  }
}
// 4 bit: one operand per word.
__device__ inline void extract4(uint32_t w, uintx4& a) {
  const uint32_t w8 = w >> 8;
  a[0] = w & 0x000F000Fu;
  a[1] = w & 0x00F000F0u;
  a[2] = w8 & 0x000F000Fu;
  a[3] = w8 & 0x00F000F0u;
}

constexpr int kEK = 4;             // query-side operands carry 2^kEK
constexpr int kEP = 6;             // weight-side operands carry 2^kEP
constexpr float kHeadroom = 4.0f;  // lazy rescale: weights may reach 2^kHeadroom
constexpr int kWaves = 8;          // waves per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kTailTok = kThreads / 4;  // fp16-tail tokens per pass (4 threads per token)
constexpr int kTailEntry = kWaves;
constexpr int kBkStride = 80;      // words per head row of the query-side operand in LDS  // slot of the fp16 tail in the workgroup merge

// Everything one wave loads for one 32-token group (held in registers so that the
// next group's loads are in flight while the current one is computed).
template <int BITS>
struct GroupRegs {
  uint32_t kw[2 * BITS], vw[2 * BITS];  // packed codes: one (2 bit) or two (4 bit) 128-bit loads each
  uint32_t ks2, kz2;                    // K scaler / zero-point of channels 2*lane, 2*lane+1
  uintx4 sv, zv;                        // V scalers (column's u) and zero-points (row's u) of 8 tokens
};

template <int BITS>
__device__ inline void load_group(GroupRegs<BITS>& g, const MfmaParams& p, size_t grp, int lane, int us, int rb,
                                  int zrow_ld) {
  constexpr int NWORDS = TKV_D * BITS;
  const uint32_t* kc = p.k_codes + grp * NWORDS;
  const uint32_t* vc = p.v_codes + grp * NWORDS;
#pragma unroll
  for (int x = 0; x < BITS / 2; ++x) {
    const uintx4 t = *reinterpret_cast<const uintx4*>(kc + 256 * x + 4 * lane);
    const uintx4 u = *reinterpret_cast<const uintx4*>(vc + 256 * x + 4 * lane);
#pragma unroll
    for (int y = 0; y < 4; ++y) {
      g.kw[4 * x + y] = t[y];
      g.vw[4 * x + y] = u[y];
    }
  }
  g.ks2 = reinterpret_cast<const uint32_t*>(p.k_scale + grp * TKV_D)[lane];
  g.kz2 = reinterpret_cast<const uint32_t*>(p.k_zero + grp * TKV_D)[lane];
  g.sv = *reinterpret_cast<const uintx4*>(p.v_scale + (grp * 4 + us) * TKV_G + 8 * rb);
  g.zv = *reinterpret_cast<const uintx4*>(p.v_zero + (grp * 4 + zrow_ld) * TKV_G + 8 * rb);
}

struct MergeSmem {
  float m[kWaves + 1][4];
  float l[kWaves + 1][4];
  float z[kWaves][4][4];
  float o[kWaves + 1][4][TKV_D];
};

// fp16 tail (ring of unquantized tokens) of one KV head, computed by the whole workgroup
// with plain float math; result goes to entry kTailEntry of the merge arrays.
__device__ inline void tail_attention(const MfmaParams& p, MergeSmem& ms, float (*q_s)[TKV_D], float (*x_s)[kThreads],
                                      float (*w_s)[4], size_t bh, int nq, int n, int G) {
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int ring = p.residual + TKV_G;
  const int r_total = n - nq;
  bool first = true;
  for (int sb0 = 0; sb0 < r_total; sb0 += kTailTok) {
    const int cnt = min(kTailTok, r_total - sb0);
    // phase 1: logits; 4 threads per token, each over 32 channels, combined by shuffles
    const int tk = tid / 4, part = tid % 4;  // token in sub-block, channel quarter
    float x[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    {
      const int tok = nq + sb0 + min(tk, cnt - 1);
      const uintx4* krow = reinterpret_cast<const uintx4*>(p.k_resid + (bh * ring + (size_t)(tok % ring)) * TKV_D) + 4 * part;
      uintx4 kv[4];
#pragma unroll
      for (int c8 = 0; c8 < 4; ++c8) kv[c8] = krow[c8];
      float a[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c8 = 0; c8 < 4; ++c8) {
#pragma unroll
        for (int y = 0; y < 4; ++y) {
          const uint32_t w = kv[c8][y];
          const half2_t k2 = as_half2(w);
          const float k0 = (float)k2[0], k1 = (float)k2[1];
          const int c = 32 * part + 8 * c8 + 2 * y;
#pragma unroll
          for (int hh = 0; hh < 4; ++hh) {
            a[hh] = __builtin_fmaf(q_s[hh][c], k0, a[hh]);
            a[hh] = __builtin_fmaf(q_s[hh][c + 1], k1, a[hh]);
          }
        }
      }
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) {
        a[hh] += __shfl_xor(a[hh], 1, 64);
        a[hh] += __shfl_xor(a[hh], 2, 64);
        if (tk < cnt) x[hh] = a[hh] * p.scale2;
      }
    }
    // phase 2: workgroup max and weights
    float wm[4];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      float v = x[hh];
      for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
      wm[hh] = v;
    }
    if (lane == 0)
      for (int hh = 0; hh < 4; ++hh) w_s[wave][hh] = wm[hh];
    __syncthreads();
    float mx[4], pw[4];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      float v = w_s[0][hh];
      for (int w = 1; w < kWaves; ++w) v = fmaxf(v, w_s[w][hh]);
      mx[hh] = v;  // finite: the sub-block holds at least one token
      pw[hh] = tk < cnt ? exp2f(x[hh] - v) : 0.f;
      if (part == 0) x_s[hh][tk] = pw[hh];
    }
    __syncthreads();
    // phase 3: weighted V sum; thread = (channel pair, token residue class)
    float acc[4][2] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};
    float ls[4] = {0.f, 0.f, 0.f, 0.f};
    // every wave takes tokens wave, wave + 8, ...; all of its rows (<= 16) are loaded before
    // the first is used (rows past the end re-read the last one with weight 0)
    {
      constexpr int RW = kTailTok / kWaves;  // 16
      uint32_t v2[RW];
#pragma unroll
      for (int y = 0; y < RW; ++y) {
        const int tok = nq + sb0 + min(wave + y * kWaves, cnt - 1);
        v2[y] = reinterpret_cast<const uint32_t*>(p.v_resid + (bh * ring + (size_t)(tok % ring)) * TKV_D)[lane];
      }
#pragma unroll
      for (int y = 0; y < RW; ++y) {
        const int t = wave + y * kWaves;
        const half2_t vv = as_half2(v2[y]);
        const float v0 = (float)vv[0], v1 = (float)vv[1];
#pragma unroll
        for (int hh = 0; hh < 4; ++hh) {
          const float pp = t < cnt ? x_s[hh][t] : 0.f;
          acc[hh][0] = __builtin_fmaf(pp, v0, acc[hh][0]);
          acc[hh][1] = __builtin_fmaf(pp, v1, acc[hh][1]);
          ls[hh] += pp;
        }
      }
    }
    // reduce over the 8 waves through the (still unused) per-wave merge slots
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      ms.o[wave][hh][2 * lane] = acc[hh][0];
      ms.o[wave][hh][2 * lane + 1] = acc[hh][1];
      if (lane == 0) ms.l[wave][hh] = ls[hh];
    }
    __syncthreads();
    {
      const int hh = tid / TKV_D, c = tid % TKV_D;  // 512 threads = 4 heads x 128 channels
      float O = 0.f, L = 0.f;
      for (int w = 0; w < kWaves; ++w) {
        O += ms.o[w][hh][c];
        L += ms.l[w][hh];
      }
      if (first) {
        ms.o[kTailEntry][hh][c] = O;
        if (c == 0) {
          ms.m[kTailEntry][hh] = mx[hh];
          ms.l[kTailEntry][hh] = L;
        }
      } else {
        const float mo = ms.m[kTailEntry][hh], mn = fmaxf(mo, mx[hh]);
        const float a_old = exp2f(mo - mn), a_new = exp2f(mx[hh] - mn);
        ms.o[kTailEntry][hh][c] = ms.o[kTailEntry][hh][c] * a_old + O * a_new;
        __syncthreads();  // every channel has read the old max before it is replaced
        if (c == 0) {
          ms.l[kTailEntry][hh] = ms.l[kTailEntry][hh] * a_old + L * a_new;
          ms.m[kTailEntry][hh] = mn;
        }
      }
    }
    first = false;
    __syncthreads();
  }
  (void)G;
}

template <int BITS>
__global__ __launch_bounds__(kThreads) void quant_attn_mfma_kernel(MfmaParams p) {
  // per wave: query-side operand [hi/lo][4 heads][128 ch] fp16 + zero-points [128] fp16
  // head rows are padded from 64 to 80 words: the 16 (head, k-block) operand reads of one
  // ds_read_b128 then fall into 16 different 16-byte bank groups
  __shared__ __attribute__((aligned(16))) uint32_t bk_s[kWaves][2][4][kBkStride];
  __shared__ __attribute__((aligned(16))) uint32_t kz_s[kWaves][TKV_D / 2];
  __shared__ MergeSmem ms;
  __shared__ float q_s[4][TKV_D];
  __shared__ float x_s[4][kThreads];
  __shared__ float w_s[kWaves][4];
  __shared__ int s_next;

  const int b = blockIdx.z, h = blockIdx.y, chunk = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);  // wave-uniform: keeps group addresses scalar
  const int G = p.hq / p.hkv;
  const int n = p.lens.n[b];
  const int nq = tkv::n_quantized(n, p.residual);
  const int jq = nq / TKV_G;
  const size_t bh = (size_t)b * p.hkv + h;
  const size_t grp_base = bh * (size_t)(p.capacity / TKV_G);
  // Work split of this sequence: the tail counts as (n - nq)/4 groups and belongs to
  // the last chunk, so that chunk gets correspondingly fewer quantized groups.
  const bool has_tail = chunk == p.n_chunks - 1;
  const int tail_equiv = (n - nq + 7) / 8;
  const int gpc = max(1, (jq + tail_equiv + p.n_chunks - 1) / p.n_chunks);
  const int blk0 = min(chunk * gpc, jq);
  const int blk1 = has_tail ? jq : min(blk0 + gpc, jq);

  long long ts[8];
  ts[0] = wall_clock64();
  const int slot = lane % 16, rb = lane / 16;
  const int hs = slot % 4, us = slot / 4;  // this lane's operand column: head, channel group
  const __half* qrow = p.q + ((size_t)b * p.hq + (size_t)h * G) * TKV_D;

  if (tid == 0) s_next = blk0 + 2 * kWaves;
  __syncthreads();
  if (has_tail) {
    for (int i = tid; i < 4 * TKV_D; i += kThreads) {
      const int hh = i / TKV_D, c = i % TKV_D;
      q_s[hh][c] = hh < G ? __half2float(qrow[(size_t)hh * TKV_D + c]) : 0.f;
    }
  }

  // query as exact fp16 B operand (zero-point term) and as scaled float (scaler term)
  uintx4 bq[4];
#pragma unroll
  for (int m = 0; m < 4; ++m)
    bq[m] = *reinterpret_cast<const uintx4*>(qrow + (size_t)(hs < G ? hs : G - 1) * TKV_D + 32 * m + 8 * rb);
  if (hs >= G) {
#pragma unroll
    for (int m = 0; m < 4; ++m) bq[m] = uintx4{0u, 0u, 0u, 0u};
  }
  // K-prep role: this lane owns channels 2*lane, 2*lane+1; their field position is lane%4
  // (2 bit: 4^pos) or lane%2 (4 bit: 16^pos).
  float qf[4][2];
  {
    const int pos = BITS == 2 ? lane % 4 : lane % 2;
    const float comp = BITS == 2 ? (float)(1 << kEK) / (float)(1 << (2 * pos)) : (float)(1 << kEK) / (float)(1 << (4 * pos));
    uint32_t q2[4];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh)  // heads >= G re-read head G-1 (in bounds) and are zeroed below
      q2[hh] = reinterpret_cast<const uint32_t*>(qrow + (size_t)(hh < G ? hh : G - 1) * TKV_D)[lane];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      const half2_t qq = as_half2(q2[hh]);
      qf[hh][0] = hh < G ? (float)qq[0] * comp : 0.f;
      qf[hh][1] = hh < G ? (float)qq[1] * comp : 0.f;
    }
  }
  // codes carry 2^-24, query side 2^kEK, so S = acc * 2^(24-kEK)
  const float K1 = p.scale2 * (float)(1 << (24 - kEK));

  floatx4 acc_o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc_o[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  floatx4 acc_z = {0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY;

  // A operand of the z_v / denominator MFMA: rows 0..3 hold z_v[u = row] (loaded per group)
  // times the constant that undoes the weight-side scaling, row 4 holds that constant
  // alone (denominator), rows 5.. are zero.  Built branch-free as load * zmul + zadd.
  const int zrow = slot;                   // as A operand this lane holds row `slot`
  const int zrow_ld = zrow < 4 ? zrow : 3;  // rows >= 4 load a valid row and multiply it by 0
  half2_t zmul[4], zadd[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    // element k = 2j + e of this lane carries 2^-kEP * (4^j | 16^(j%2))
    const float w = BITS == 2 ? (float)(1 << (2 * j)) / (float)(1 << kEP) : (float)(1 << (4 * (j % 2))) / (float)(1 << kEP);
    const _Float16 wm = (_Float16)(zrow < 4 ? w : 0.f), wa = (_Float16)(zrow == 4 ? w : 0.f);
    zmul[j] = half2_t{wm, wm};
    zadd[j] = half2_t{wa, wa};
  }
  // exponent offsets that put 2^kEP / (4^j | 16^(j%2)) into the weights; value i of the
  // lane (tile tau = i/4, row x = i%4) is element kappa = 4 tau + x, register j = kappa/2
  float off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int j = i / 2;
    off[i] = BITS == 2 ? (float)(kEP - 2 * j) : (float)(kEP - 4 * (j % 2));
  }

  // One group's worth of work for this wave; `cur` was loaded two iterations earlier.
  auto process = [&](const GroupRegs<BITS>& cur) {
    // ---- query-side operand of this group: (q s) split into hi + lo, through LDS
    {
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) {
        const uint32_t hi = mix_hi_pair(qf[hh][0], qf[hh][1], cur.ks2);  // products are exact in float32
        bk_s[wave][0][hh][lane] = hi;
        bk_s[wave][1][hh][lane] = mix_lo_pair(qf[hh][0], qf[hh][1], cur.ks2, hi);
      }
      kz_s[wave][lane] = cur.kz2;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- zero-point term: cz[slot] = sum_c z[c] q[c], identical in every row
    floatx4 acc_cz = {0.f, 0.f, 0.f, 0.f};
    {
      uintx4 az[4];
#pragma unroll
      for (int m = 0; m < 4; ++m) az[m] = *reinterpret_cast<const uintx4*>(&kz_s[wave][(32 * m + 8 * rb) / 2]);
#pragma unroll
      for (int m = 0; m < 4; ++m) acc_cz = mfma(az[m], bq[m], acc_cz);
    }
    // ---- scaler term for the two 16-token tiles
    floatx4 acc_s[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int m2 = 0; m2 < 2; ++m2) {  // pairs of MFMA steps m = 2*m2, 2*m2+1
      uintx4 bh2[2], bl2[2];
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        const int m = 2 * m2 + y;
        bh2[y] = *reinterpret_cast<const uintx4*>(&bk_s[wave][0][hs][(32 * m + 8 * rb) / 2]);
        bl2[y] = *reinterpret_cast<const uintx4*>(&bk_s[wave][1][hs][(32 * m + 8 * rb) / 2]);
      }
#pragma unroll
      for (int tau = 0; tau < 2; ++tau) {
        uintx4 a[2];
        if (BITS == 2) {
          extract<2>(cur.kw[2 * tau + m2], a[0], a[1]);
        } else {
          extract4(cur.kw[4 * tau + 2 * m2], a[0]);
          extract4(cur.kw[4 * tau + 2 * m2 + 1], a[1]);
        }
#pragma unroll
        for (int y = 0; y < 2; ++y) {
          acc_s[tau] = mfma(a[y], bh2[y], acc_s[tau]);
          acc_s[tau] = mfma(a[y], bl2[y], acc_s[tau]);
        }
      }
    }

    // ---- online softmax (log2 domain), lazy rescale
    const float cz = acc_cz[0] * p.scale2;
    const float mx = fmaxf(fmaxf(fmaxf(acc_s[0][0], acc_s[0][1]), fmaxf(acc_s[0][2], acc_s[0][3])),
                           fmaxf(fmaxf(acc_s[1][0], acc_s[1][1]), fmaxf(acc_s[1][2], acc_s[1][3])));
    const float xmax = __builtin_fmaf(mx, K1, cz);  // largest logit among this lane's 8 tokens
    if (__builtin_amdgcn_ballot_w64(xmax - m_run > kHeadroom) != 0ull) {
      // new reference maximum, uniform over the lanes that share a query head
      float mn = fmaxf(m_run, xmax);
      mn = fmaxf(mn, __shfl_xor(mn, 4, 64));
      mn = fmaxf(mn, __shfl_xor(mn, 8, 64));
      mn = fmaxf(mn, __shfl_xor(mn, 16, 64));
      mn = fmaxf(mn, __shfl_xor(mn, 32, 64));
      const float alpha = exp2f(m_run - mn);  // 0 on the first group
#pragma unroll
      for (int i = 0; i < 8; ++i) acc_o[i] *= alpha;
      acc_z *= alpha;
      m_run = mn;
    }
    const float czm = cz - m_run;
    float pw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pw[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(acc_s[i / 4][i % 4], K1, czm + off[i]));

    // ---- weight-side operands: p*s_v (hi, lo) and p (hi, lo)
    uintx4 b2h, b2l, bph, bpl, a_zv;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t svj = cur.sv[j];
      const float w0 = pw[2 * j], w1 = pw[2 * j + 1];
      b2h[j] = mix_hi_pair(w0, w1, svj);
      b2l[j] = mix_lo_pair(w0, w1, svj, b2h[j]);
      bph[j] = pack2((_Float16)w0, (_Float16)w1);
      bpl[j] = residual_pair(w0, w1, bph[j]);
      const uint32_t zvj = cur.zv[j];
      const half2_t t = __builtin_elementwise_fma(as_half2(zvj), zmul[j], zadd[j]);
      a_zv[j] = __builtin_bit_cast(uint32_t, t);
    }
    acc_z = mfma(a_zv, bph, acc_z);
    acc_z = mfma(a_zv, bpl, acc_z);

    // ---- P.V: 8 blocks of 16 channels
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) {
      uintx4 a[2];
      if (BITS == 2) {
        extract<2>(cur.vw[wd], a[0], a[1]);
      } else {
        extract4(cur.vw[(wd / 2) * 4 + 2 * (wd % 2)], a[0]);
        extract4(cur.vw[(wd / 2) * 4 + 2 * (wd % 2) + 1], a[1]);
      }
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        acc_o[2 * wd + y] = mfma(a[y], b2h, acc_o[2 * wd + y]);
        acc_o[2 * wd + y] = mfma(a[y], b2l, acc_o[2 * wd + y]);
      }
    }
    __builtin_amdgcn_wave_barrier();
  };

  ts[1] = wall_clock64();
  // Three-deep register ring: while one group is computed the wave's next two groups are in
  // flight.  After a static first round the waves of a workgroup draw their groups from a
  // shared LDS counter: the two waves that share a SIMD do not progress evenly, and with a
  // static split the slower one ran alone (and poorly overlapped) for the last third.
  {
    GroupRegs<BITS> r0, r1, r2;
    const int last = p.dbg_mode == 1 ? blk0 : blk1 - 1;  // loads past the chunk are clamped to its last group and ignored
    auto grab = [&]() -> int {
      int v = 0;
      if (lane == 0) v = atomicAdd(&s_next, 1);
      return __builtin_amdgcn_readfirstlane(v);
    };
    int i0 = blk0 + wave, i1 = blk0 + kWaves + wave, i2;
    if (i0 < blk1) {
      load_group<BITS>(r0, p, grp_base + min(i0, last), lane, us, rb, zrow_ld);
      load_group<BITS>(r1, p, grp_base + min(i1, last), lane, us, rb, zrow_ld);
      for (;;) {
        i2 = grab();
        load_group<BITS>(r2, p, grp_base + min(i2, last), lane, us, rb, zrow_ld);
        process(r0);
        if (i1 >= blk1) break;
        i0 = grab();
        load_group<BITS>(r0, p, grp_base + min(i0, last), lane, us, rb, zrow_ld);
        process(r1);
        if (i2 >= blk1) break;
        i1 = grab();
        load_group<BITS>(r1, p, grp_base + min(i1, last), lane, us, rb, zrow_ld);
        process(r2);
        if (i0 >= blk1) break;
      }
    }
  }
  ts[2] = wall_clock64();
  __syncthreads();
  ts[3] = wall_clock64();
  if (has_tail && n > nq) {
    tail_attention(p, ms, q_s, x_s, w_s, bh, nq, n, G);
  } else if (tid < 4) {
    ms.m[kTailEntry][tid] = -INFINITY;
    ms.l[kTailEntry][tid] = 0.f;
  }
  __syncthreads();

  ts[4] = wall_clock64();
  // ---- per-wave results -> LDS.  acc_z rows: lanes 0..15 (rb 0) hold rows 0..3 = z-terms
  // for u = row; lanes 16..31 register 0 hold row 4 = denominator.
  if (rb == 0) {
#pragma unroll
    for (int x = 0; x < 4; ++x)
      if (x == us) ms.z[wave][hs][us] = acc_z[x];
    if (us == 0) ms.m[wave][hs] = m_run;
  }
  if (rb == 1 && us == 0) ms.l[wave][hs] = acc_z[0];
  __syncthreads();
  {
    const float zt = ms.z[wave][hs][us];
    const float unscale = (float)(1 << (24 - kEP));
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
      if (cb / 2 == us) {
#pragma unroll
        for (int x = 0; x < 4; ++x) ms.o[wave][hs][16 * cb + 4 * rb + x] = __builtin_fmaf(acc_o[cb][x], unscale, zt);
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < G * TKV_D; i += kThreads) {
    const int hh = i / TKV_D, c = i % TKV_D;
    float M = -INFINITY;
    for (int w = 0; w <= kWaves; ++w) M = fmaxf(M, ms.m[w][hh]);
    float L = 0.f, O = 0.f;
    for (int w = 0; w <= kWaves; ++w) {
      const float mw = ms.m[w][hh];
      if (mw == -INFINITY) continue;
      const float wgt = exp2f(mw - M);
      L += ms.l[w][hh] * wgt;
      O += ms.o[w][hh][c] * wgt;
    }
    float* dst = p.parts + (((size_t)b * p.hq + (size_t)h * G + hh) * p.n_chunks + chunk) * TKV_PART_STRIDE;
    // device-scope stores: visible to the merging workgroup without a cache write-back
    __hip_atomic_store(dst + 2 + c, O, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (c == 0) {
      __hip_atomic_store(dst, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(dst + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- the last workgroup of this (sequence, KV head) to arrive merges all chunks.
  // Partials travel through device-scope (cache-bypassing) stores and loads, ordered by
  // waiting for the stores to complete before the arrival counter is bumped: a release /
  // acquire fence pair would write back and invalidate the whole L2 (tens of microseconds).
  ts[5] = wall_clock64();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  ts[6] = wall_clock64();
  if (p.dbg_ts && lane == 0) {
    long long* d = p.dbg_ts + ((((size_t)b * p.hkv + h) * p.n_chunks + chunk) * kWaves + wave) * 8;
    for (int i = 0; i < 7; ++i) d[i] = ts[i];
  }
  if (tid == 0) w_s[0][0] = __uint_as_float(atomicAdd(&p.arrivals[bh], 1u) == (uint32_t)(p.n_chunks - 1) ? 1u : 0u);
  __syncthreads();
  if (__float_as_uint(w_s[0][0]) == 0u) return;
  if (tid == 0) p.arrivals[bh] = 0u;
  if (tid < G * TKV_D) {
    const int hh = tid / TKV_D, c = tid % TKV_D;
    const size_t head = (size_t)b * p.hq + (size_t)h * G + hh;
    const float* base = p.parts + head * p.n_chunks * TKV_PART_STRIDE;
    float M = -INFINITY;
    auto ld = [](const float* ptr) { return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
#pragma unroll 8
    for (int k = 0; k < p.n_chunks; ++k) M = fmaxf(M, ld(base + (size_t)k * TKV_PART_STRIDE));
    float L = 0.f, O = 0.f;
#pragma unroll 8
    for (int k = 0; k < p.n_chunks; ++k) {
      const float* pk = base + (size_t)k * TKV_PART_STRIDE;
      const float mk = ld(pk);
      const float w = mk == -INFINITY ? 0.f : exp2f(mk - M);
      L = __builtin_fmaf(ld(pk + 1), w, L);
      O = __builtin_fmaf(ld(pk + 2 + c), w, O);
    }
    p.out[head * TKV_D + c] = __float2half_rn(L > 0.f ? O / L : 0.f);
  }
}

}  // namespace

namespace tkv {
void* g_mfma_dbg = nullptr;

int32_t launch_quant_attn_mfma(const tkv_quant_desc* d, const tkv_quant_cache* c, const __half* q, __half* out,
                               float scale2, float* parts, uint32_t* arrivals, int n_chunks,
                               const TkvSeqLens& lens, hipStream_t s) {
  if (d->head_dim != TKV_D || d->group_size != TKV_G) return TKV_E_UNSUPPORTED;
  if (d->n_q_heads / d->n_kv_heads > 4) return TKV_E_UNSUPPORTED;
  MfmaParams p;
  p.k_codes = (const uint32_t*)c->k_codes;
  p.v_codes = (const uint32_t*)c->v_codes;
  p.k_scale = (const __half*)c->k_scale;
  p.k_zero = (const __half*)c->k_zero;
  p.v_scale = (const __half*)c->v_scale;
  p.v_zero = (const __half*)c->v_zero;
  p.k_resid = (const __half*)c->k_resid;
  p.v_resid = (const __half*)c->v_resid;
  p.q = q;
  p.parts = parts;
  p.arrivals = arrivals;
  p.out = out;
  p.scale2 = scale2;
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.residual = d->residual;
  p.capacity = d->capacity;
  p.n_chunks = n_chunks;
  p.dbg_ts = (long long*)g_mfma_dbg;
  p.dbg_mode = getenv("TKV_DEBUG_MODE") ? atoi(getenv("TKV_DEBUG_MODE")) : 0;
  p.lens = lens;
  const dim3 grid(n_chunks, d->n_kv_heads, d->batch);
  if (d->bits == 2)
    quant_attn_mfma_kernel<2><<<grid, kThreads, 0, s>>>(p);
  else if (d->bits == 4)
    quant_attn_mfma_kernel<4><<<grid, kThreads, 0, s>>>(p);
  else
    return TKV_E_UNSUPPORTED;
  return launch_status();
}

}  // namespace tkv

extern "C" void tkv_debug_set_dump(void* ptr) { tkv::g_mfma_dbg = ptr; }
