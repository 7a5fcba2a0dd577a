// Matrix-core kernel of tkv_quant_attn_decode (Sec. 2.1 Eq. 3 over the quantized cache
// of Sec. 4.3) for gfx950, 4 query heads of a KV head per workgroup, D = 128, bits 1, 2 or 4, quantization group 32
// or 64 (Sec. 5.1 runs 1 and 2 bits with groups of 64).
//
// One wave64 owns one packed block of 32 tokens at a time (half a key group when the
// quantization group is 64; "group" below means such a block).  Both contractions run on
// v_mfma_f32_16x16x32_f16 with the packed codes as the A operand:
//
//   * a b-bit code c sitting at mantissa bits [bp, bp+b) of an otherwise zero fp16 IS
//     the subnormal number c * 2^bp * 2^-24, so one v_and_b32 per register turns two
//     codes into two exact fp16 operands (no bias, no convert); the 2^bp factor is
//     compensated in the other operand;
//   * q.K-hat = sum_c code[t][c] * (q[c] s[c]) + sum_c q[c] z[c]: the scaler moves into
//     the query operand, split into fp16 hi + lo parts so the product keeps ~22 bits.
//     The 16 operand columns are 4 query heads x 4 column groups; even groups carry the hi
//     part and odd groups the lo part, so ONE MFMA per (16 tokens, 32 channels) produces
//     both partial sums and a single cross-lane add joins them.  The zero-point term does
//     not depend on the token: it is computed once per workgroup for all of its groups
//     (16 groups per MFMA) and kept in an LDS table;
//   * p.V-hat = sum_t code[t][d] * (p[t] s_v[t][u]) + sum_t p[t] z_v[t][u]: here the 4
//     column groups are the 4 channel groups u, so the weights never leave the lanes that
//     produced them (the D layout of the first product is the B layout of the second);
//     z_v and the softmax denominator ride on one more MFMA.  The weights go in as one
//     fp16 number each (the product p s_v is rounded once).
//
// The machine issues one vector or matrix instruction per SIMD at a time and a wave issues
// in order, so the cost of a group is close to the plain sum of its instructions: the
// design minimises instruction count first, then hides latencies with three resident
// waves per SIMD (2 bit) and a three-deep ring of direct global->LDS loads per wave.
//
// Softmax is online per wave with lazy rescaling; the waves of a workgroup and the chunks
// of a sequence are merged with log-sum-exp merges, the last workgroup of a (sequence, KV
// head) to finish doing the cross-chunk merge.
#include "tkv_common.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
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
  float* parts;        // sequence after sequence: [Hq][chunks of the sequence][D + 4]
  uint32_t* arrivals;  // [B][Hkv * quarters of a group], zero between calls
  __half* out;         // [B][Hq][D]
  float scale2;
  int32_t hq, hkv, residual, capacity;
  int32_t batch;
#ifdef TKV_PHASE
  long long* prof;  // phase time stamps (profiling builds only)
#endif
  TkvSeqLens lens;
  TkvSeqLens chunks;  // split-K chunks of every sequence, in proportion to its length: blockIdx.x runs over all of them
  // The step's new tokens, when the call also appends them (Eq. 2): the last n_add[b] tokens of
  // sequence b, rows k_new / v_new [B][n_stride][Hkv][D], are copied into the fp16 ring by the
  // workgroups that own the head's tail before they read it.  k_new == nullptr: none.
  const __half* k_new;
  const __half* v_new;
  int32_t n_stride;
  TkvSeqLens n_add;
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

// v + (value of the lane 4 places away in the same row of 16 lanes)
__device__ inline float ror4_add(float v) {
  const int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124 /* row_ror:4 */, 0xF, 0xF, false);
  return v + __builtin_bit_cast(float, r);
}

// fp16 hi/lo split of a product, written so that each part is one fused multiply-add
// with an fp16 result (the compiler selects v_fma_mixlo/mixhi_f16 for this shape):
//   hi = f16(a * b), lo = f16(a * b - hi)   (the FMA makes the residual exact)
// s2 holds two fp16 scalers; the results are packed the same way.  No inline assembly:
// operands that come straight from MFMA / transcendental results have read hazards that
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

// 1 bit: four MFMA operands out of one word.  Operands 1 and 3 sit four mantissa bits
// higher than operands 0 and 2: their results carry an extra 2^4.
__device__ inline void extract1(uint32_t w, uintx4 (&a)[4]) {
  const uint32_t w8 = w >> 8;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    a[0][j] = w & (0x00010001u << j);
    a[1][j] = w & (0x00100010u << j);
    a[2][j] = w8 & (0x00010001u << j);
    a[3][j] = w8 & (0x00100010u << j);
  }
}
// 2 bit: two MFMA operands (8 registers) out of one 32-bit word of packed codes.
__device__ inline void extract2(uint32_t w, uintx4& a0, uintx4& a1) {
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
// 4 bit: one operand per word.
__device__ inline void extract4(uint32_t w, uintx4& a) {
  const uint32_t w8 = w >> 8;
  a[0] = w & 0x000F000Fu;
  a[1] = w & 0x00F000F0u;
  a[2] = w8 & 0x000F000Fu;
  a[3] = w8 & 0x00F000F0u;
}

__device__ inline void lds_load16(const void* g, void* l) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}
__device__ inline void lds_load4(const void* g, void* l) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)l, 4, 0, 0);
}

// Query-side operands q s 2^(kEK - position shift) are fp16 hi + lo pairs.  kEK = 0 leaves the
// whole fp16 range to the product of query and key scaler; the parts that then fall into
// fp16's subnormal range keep an absolute precision (2^-25 per operand) that is worth less
// than 1e-5 in the logit, so nothing is gained by a larger kEK (measured 0 to 4).
constexpr int kEK = 0;
// Weight-side operands carry 2^kEP: fp16 weights p 2^(kEP - position shift) (p up to
// 2^kHeadroomLog2) times the value scaler must stay below 65504, and so must the zero-point
// times 2^(position shift - kEP).  kEP = 2 keeps both finite for value magnitudes up to about
// 1000 at every bit width; the attention error does not depend on it (measured 0 to 6).
constexpr int kEP = 2;
constexpr int kHeadroomLog2 = 4;  // lazy rescale: weights may reach 2^kHeadroomLog2
constexpr int kRefBelowMax = 3;   // a rescale puts the reference this far under the largest logit (< headroom)
constexpr int kBkStride = 80;     // words per head row of the query-side operand in LDS
constexpr int kMaxGpc = 512;      // groups per chunk that the zero-point table holds
constexpr int kTailWaves = 4;     // waves of the last chunk that share the fp16 tail

struct TailEntry {
  float m[4];
  float l[4];
  float o[4][TKV_D];
};
// Results of one wave for the merge inside the workgroup; it takes the place of the start of
// the wave's own load ring once the wave has left the group loop.
struct MergeWave {
  float m[4];
  float l[4];
  float z[4][4];
  float o[4][TKV_D];
};

// ---- LDS plan (dynamic shared memory) ---------------------------------------------------
//   bk     per wave [hi/lo][4 heads][80 words]: query-side operands of the next group
//   ring   per wave 3 K slots (codes, scalers) then 3 V slots (codes, scalers, zero-points);
//          the direct global->LDS loads put lane l's bytes at slot + 16*l (codes) or
//          slot + 4*l (fp16 rows), i.e. a slot is a copy of the group's packed block.  After
//          the main loop the start of a wave's ring holds its results for the workgroup merge.
//   cz     zero-point term of every group of the chunk, [group][4 heads] float
//   tail   partial results of the waves that share the fp16 tail
//   q      the 4 query rows as fp16, for the tail
// GS = quantization group / 32: the K scalers of a slot are those of the block's key group,
// the V scalers and zero-points [128 / (32 GS)][32 tokens] fp16 each.
template <int BITS, int GS, int W>
struct Cfg {
  static constexpr int kThreads = 64 * W;
  static constexpr int kCode = 512 * BITS;  // bytes of K (or V) codes of one block
  static constexpr int kKPart = kCode + 256;
  static constexpr int kVPart = kCode + 512;
  static constexpr int oVs = kCode;                 // V scalers inside a V slot
  static constexpr int oVz = kCode + 256 / GS;      // V zero-points
  static constexpr int kDepth = 3;
  static constexpr int kWaveRing = kDepth * (kKPart + kVPart);
  // direct-to-LDS load instructions per part: 1 bit = two 4-byte-per-lane loads of codes, else
  // 16-byte-per-lane loads; GS = 2 fetches V scalers and zero-points with one instruction
  static constexpr int kCodeLoads = BITS == 1 ? 2 : BITS / 2;
  static constexpr int kKLoads = kCodeLoads + 1;
  static constexpr int kVLoads = kCodeLoads + (GS == 1 ? 2 : 1);
  static constexpr int kCodeWords = BITS == 1 ? 2 : 2 * BITS;  // code words per lane and part
  static constexpr int kBkWave = 2 * 4 * kBkStride * 4;
  static constexpr int oRing = W * kBkWave;
  static constexpr int oCz = oRing + W * kWaveRing;
  static constexpr int oTail = oCz + kMaxGpc * 16;
  static constexpr int oQ = oTail + kTailWaves * (int)sizeof(TailEntry);
  static constexpr int kLdsBytes = oQ + 4 * TKV_D * 2;
  static_assert(sizeof(MergeWave) <= (size_t)kWaveRing, "a wave's results fit in its own ring");
  static_assert((3 * 4 * TKV_MAX_CHUNKS + 4 * 4 * TKV_D + 4) * 4 <= (size_t)W * kWaveRing, "merge scratch must fit in the ring");
  static_assert(kLdsBytes + 64 <= 160 * 1024, "LDS budget of one compute unit");
};

// fp16 tail (ring of unquantized tokens): wave w of the last chunk takes the 32-token
// sub-blocks w, w + kTailWaves, ... with plain float math and an online softmax, and leaves
// its partial result in `te`.  Lane = (token, channel half) for the logits, lane = channel
// pair for the weighted sum.
__device__ inline void tail_wave(const MfmaParams& p, TailEntry& te, const uint32_t* q_h, size_t bh, int nq, int n,
                                 int ring, int wave, int lane) {
  const int r_total = n - nq;
  const int t = lane / 2, half = lane % 2;
  float M[4], Ls[4], acc[4][2];
#pragma unroll
  for (int hh = 0; hh < 4; ++hh) M[hh] = -INFINITY, Ls[hh] = 0.f, acc[hh][0] = 0.f, acc[hh][1] = 0.f;
  for (int sb = wave; sb * 32 < r_total; sb += kTailWaves) {
    const int cnt = min(32, r_total - 32 * sb);
    const int t0 = nq + 32 * sb;
    float x[4];
    {
      const int tok = t0 + min(t, cnt - 1);
      const uintx4* krow = reinterpret_cast<const uintx4*>(p.k_resid + (bh * ring + (size_t)(tok % ring)) * TKV_D + 64 * half);
      uintx4 kv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) kv[i] = krow[i];
      __builtin_amdgcn_sched_barrier(0);  // all eight loads in flight before the first is used
      float a[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
#pragma unroll
        for (int hh = 0; hh < 4; ++hh) {
          const uintx4 q4 = *reinterpret_cast<const uintx4*>(q_h + hh * 64 + 32 * half + 4 * i);
#pragma unroll
          for (int y = 0; y < 4; ++y) {
            const uint32_t kw = kv[i][y], qw = q4[y];
            a[hh] = __builtin_amdgcn_fdot2(as_half2(kw), as_half2(qw), a[hh], false);
          }
        }
      }
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) {
        a[hh] += __shfl_xor(a[hh], 1, 64);
        x[hh] = t < cnt ? a[hh] * p.scale2 : -INFINITY;
      }
    }
    float pw[4];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      float mx = x[hh];
      for (int m = 32; m >= 2; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
      const float mn = fmaxf(M[hh], mx);  // finite: the sub-block holds at least one token
      const float alpha = exp2f(M[hh] - mn);
      pw[hh] = t < cnt ? exp2f(x[hh] - mn) : 0.f;
      float sum = half == 0 ? pw[hh] : 0.f;
      for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 64);
      Ls[hh] = Ls[hh] * alpha + sum;
      acc[hh][0] *= alpha;
      acc[hh][1] *= alpha;
      M[hh] = mn;
    }
    uint32_t v2[32];  // this lane's channel pair of every row
#pragma unroll
    for (int y = 0; y < 32; ++y) {
      const int tokv = t0 + min(y, cnt - 1);  // rows past the end re-read the last one with weight 0
      v2[y] = reinterpret_cast<const uint32_t*>(p.v_resid + (bh * ring + (size_t)(tokv % ring)) * TKV_D)[lane];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int y = 0; y < 32; ++y) {
      const half2_t vv = as_half2(v2[y]);
      const float v0 = (float)vv[0], v1 = (float)vv[1];
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) {
        const float pp = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pw[hh]), 2 * y));
        acc[hh][0] = __builtin_fmaf(pp, v0, acc[hh][0]);
        acc[hh][1] = __builtin_fmaf(pp, v1, acc[hh][1]);
      }
    }
  }
#pragma unroll
  for (int hh = 0; hh < 4; ++hh) {
    te.o[hh][2 * lane] = acc[hh][0];
    te.o[hh][2 * lane + 1] = acc[hh][1];
    if (lane == 0) te.m[hh] = M[hh], te.l[hh] = Ls[hh];
  }
}

#ifdef TKV_PHASE
#define TKV_PH()                                \
  do {                                          \
    __builtin_amdgcn_sched_barrier(0);          \
    ph[ph_n++] = wall_clock64();                \
    __builtin_amdgcn_sched_barrier(0);          \
  } while (0)
#else
#define TKV_PH() \
  do {           \
  } while (0)
#endif

template <int BITS, int GS, int W>
__global__ __launch_bounds__(64 * W) void quant_attn_mfma_kernel(MfmaParams p) {
  using C = Cfg<BITS, GS, W>;
  constexpr int KSH = GS - 1;          // key group of a block = block >> KSH
  constexpr int NU = 4 / GS;           // channel groups of a value row
  constexpr int GRP = TKV_BLK * GS;    // quantization group
  constexpr int NWORDS = TKV_D * BITS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_next;
  __shared__ uint32_t s_flag;
#ifdef TKV_PHASE
  long long ph[8];
  int ph_n = 0;
#endif
  TKV_PH();  // 0 kernel start

  // blockIdx.x counts the chunks of all sequences: which sequence, which of its chunks
  int b = 0, chunk = blockIdx.x, chunk_base = 0;
  while (b + 1 < p.batch && chunk >= p.chunks.n[b]) {
    chunk -= p.chunks.n[b];
    chunk_base += p.chunks.n[b];
    ++b;
  }
  const int n_chunks = p.chunks.n[b];
  // Groups of more than 4 query heads per KV head are served 4 heads at a time (the operand
  // columns hold 4 heads): blockIdx.y runs over (KV head, quarter of its group), and the
  // quarters of a head read the same codes.
  const int split = (p.hq / p.hkv + 3) / 4;
  const int h = blockIdx.y / split;
  const int tid = threadIdx.x, lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);  // wave-uniform: keeps group addresses scalar
  const int qh0 = h * (p.hq / p.hkv) + 4 * (blockIdx.y % split);  // first query head of this workgroup
  const int G = min(4, (h + 1) * (p.hq / p.hkv) - qh0);
  const int n = p.lens.n[b];
  const int nq = tkv::n_quantized(n, p.residual, GRP);
  const int jq = nq / TKV_BLK;
  const size_t bh = (size_t)b * p.hkv + h;
  const size_t grp_base = bh * (size_t)(p.capacity / TKV_BLK);   // first packed block of this head
  const size_t kgrp_base = bh * (size_t)(p.capacity / GRP);      // first key group
  // Work split of this sequence: a 32-token piece of the tail counts as two groups and the
  // tail belongs to the last chunk, which gets correspondingly fewer quantized groups.
  const bool has_tail = chunk == n_chunks - 1;
  const int tail_equiv = 2 * ((n - nq + 31) / 32);
  const int gpc = max(1, (jq + tail_equiv + n_chunks - 1) / n_chunks);
  const int blk0 = min(chunk * gpc, jq);
  const int blk1 = has_tail ? jq : min(blk0 + gpc, jq);
  const int last = max(blk1 - 1, blk0);  // groups past the chunk are clamped (and ignored); jq >= 1 here

  const int slot = lane % 16, rb = lane / 16;
  const int hs = slot % 4, us = slot / 4;  // this lane's operand column: head, column group
  const __half* qrow = p.q + ((size_t)b * p.hq + (size_t)qh0) * TKV_D;
  typedef uint32_t BkArr[2][4][kBkStride];
  uint32_t(*bk_s)[4][kBkStride] = reinterpret_cast<BkArr*>(smem)[wave];
  float* cz_s = reinterpret_cast<float*>(smem + C::oCz);
  TailEntry* tail_s = reinterpret_cast<TailEntry*>(smem + C::oTail);
  uint32_t* q_h = reinterpret_cast<uint32_t*>(smem + C::oQ);
  // Byte offsets (wave-uniform) of this wave's ring slots; the roles rotate every step.
  const uint32_t ring_off = C::oRing + wave * C::kWaveRing;
  const uint32_t lane16 = 16u * (uint32_t)lane, lane4 = 4u * (uint32_t)lane;  // unsigned: scalar base + 32-bit lane offset

  // ---- loads: asynchronous global -> LDS copies of a group's K part / V part ------------
  auto load_codes = [&](unsigned char* s, const unsigned char* src, uint32_t l16, uint32_t l4) {
    if (BITS == 1) {
      lds_load4(src + l4, s);
      lds_load4(src + 256 + l4, s + 256);
    } else {
#pragma unroll
      for (int x = 0; x < BITS / 2; ++x) lds_load16(src + 1024 * x + l16, s + 1024 * x);
    }
  };
  // GS = 2: lanes 0..31 fetch the block's V scalers, lanes 32..63 its zero-points (128 bytes each)
  const __half* vmeta_lane = lane < 32 ? p.v_scale + 2 * lane : p.v_zero + 2 * (lane - 32);
  auto load_kpart = [&](uint32_t so, int g) {
    const int gi = min(g, last);
    const size_t grp = grp_base + gi;
    unsigned char* s = smem + so;
    uint32_t l16 = lane16, l4 = lane4;  // opaque copies: keeps "scalar base + lane offset" addressing
    asm volatile("" : "+v"(l16), "+v"(l4));
    load_codes(s, reinterpret_cast<const unsigned char*>(p.k_codes + grp * NWORDS), l16, l4);
    lds_load4(reinterpret_cast<const unsigned char*>(p.k_scale + (kgrp_base + (gi >> KSH)) * TKV_D) + l4, s + C::kCode);
  };
  auto load_vpart = [&](uint32_t so, int g) {
    const size_t grp = grp_base + min(g, last);
    unsigned char* s = smem + so;
    uint32_t l16 = lane16, l4 = lane4;
    asm volatile("" : "+v"(l16), "+v"(l4));
    load_codes(s, reinterpret_cast<const unsigned char*>(p.v_codes + grp * NWORDS), l16, l4);
    if (GS == 1) {
      lds_load4(reinterpret_cast<const unsigned char*>(p.v_scale + grp * TKV_D) + l4, s + C::oVs);
      lds_load4(reinterpret_cast<const unsigned char*>(p.v_zero + grp * TKV_D) + l4, s + C::oVz);
    } else {
      lds_load4(vmeta_lane + grp * (TKV_D / GS), s + C::oVs);
    }
  };

  // The first three groups of a wave are fixed (wave, wave + W, wave + 2W), the rest come
  // from the workgroup's counter: their loads can start before anything else is set up.
  // ring roles: kq = K part the next QK reads, kk = K part whose scalers are prepared next,
  // kl = K slot being loaded; vp = V part of the current group, vn = the one after, vl = V
  // slot being loaded
  uint32_t kl = ring_off, kq = ring_off + C::kKPart, kk = ring_off + 2 * C::kKPart;
  uint32_t vp = ring_off + 3 * C::kKPart, vn = vp + C::kVPart, vl = vp + 2 * C::kVPart;
  const int g0 = blk0 + wave;
  int g1 = g0 + W, g2 = g0 + 2 * W;
  const bool active = g0 < blk1;
  // Set-up loads first (query rows, zero-points of this wave's first 16 groups), then the
  // ring prologue: one memory round trip covers both.
  const int ng = blk1 - blk0;
  uint32_t q2[4];   // K-prep role: this lane owns channels 2*lane, 2*lane+1
  uintx4 bq[4];     // exact fp16 query as MFMA B operand (zero-point term)
  uintx4 az[4];     // zero-point rows of 16 groups as MFMA A operand
  if (has_tail && p.k_new != nullptr) {
    // Eq. 2 in this launch: the step's new rows go into the fp16 ring (slots whose tokens were
    // quantized long ago: nothing reads them) before the workgroup's set-up barrier, behind which
    // the tail waves read the ring.  Every workgroup that reads the head's tail writes the rows
    // itself (the workgroups of a group of more than 4 query heads write the same bytes).
    const int add = p.n_add.n[b], ring = p.residual + GRP;
    for (int x = tid; x < add * 32; x += 64 * W) {
      const int i = x / 32, kv = (x % 32) / 16, part = x % 16;
      const uintx4 v = reinterpret_cast<const uintx4*>((kv ? p.v_new : p.k_new) +
                                                       (((size_t)b * p.n_stride + i) * p.hkv + h) * TKV_D)[part];
      __half* dst = const_cast<__half*>(kv ? p.v_resid : p.k_resid) + (bh * ring + (size_t)((n - add + i) % ring)) * TKV_D;
      reinterpret_cast<uintx4*>(dst)[part] = v;
    }
  }
#pragma unroll
  for (int hh = 0; hh < 4; ++hh)  // heads >= G re-read head G-1 (in bounds) and are zeroed below
    q2[hh] = reinterpret_cast<const uint32_t*>(qrow + (size_t)(hh < G ? hh : G - 1) * TKV_D)[lane];
#pragma unroll
  for (int m = 0; m < 4; ++m)
    bq[m] = *reinterpret_cast<const uintx4*>(qrow + (size_t)(hs < G ? hs : G - 1) * TKV_D + 32 * m + 8 * rb);
  auto load_az = [&](int t0) {
    const size_t grp = kgrp_base + (min(blk0 + t0 + slot, last) >> KSH);
#pragma unroll
    for (int m = 0; m < 4; ++m) az[m] = *reinterpret_cast<const uintx4*>(p.k_zero + grp * TKV_D + 32 * m + 8 * rb);
  };
  if (16 * wave < ng) load_az(16 * wave);
  __builtin_amdgcn_sched_barrier(0);
  if (active) {
    // issue order K0 V0 K1 K2 V1, then per step [K(i+3) V(i+2)]: the counter retires loads
    // in order, so "at most N outstanding" names exactly which parts have landed
    load_kpart(kl, g0);
    load_vpart(vp, g0);
    load_kpart(kq, g1);
    load_kpart(kk, g2);
    load_vpart(vn, g1);
  }
  __builtin_amdgcn_sched_barrier(0);
  if (tid == 0) s_next = blk0 + 3 * W;
  if (tid < kTailWaves * 4) {
    tail_s[tid / 4].m[tid % 4] = -INFINITY;
    tail_s[tid / 4].l[tid % 4] = 0.f;
  }
  if (tid < 4 * TKV_D / 2) {
    const int hh = tid / (TKV_D / 2);
    const uint32_t w = reinterpret_cast<const uint32_t*>(qrow + (size_t)(hh < G ? hh : G - 1) * TKV_D)[tid % (TKV_D / 2)];
    q_h[tid] = hh < G ? w : 0u;
  }

  // ---- zero-point term of every group of the chunk: cz[g][head] = scale2 * sum_c q[c] z_g[c],
  // 16 groups per MFMA (A rows = groups, B = the exact fp16 query)
  if (hs >= G) {
#pragma unroll
    for (int m = 0; m < 4; ++m) bq[m] = uintx4{0u, 0u, 0u, 0u};
  }
  for (int t0 = 16 * wave; t0 < ng; t0 += 16 * W) {
    if (t0 != 16 * wave) load_az(t0);
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int m = 0; m < 4; ++m) acc = mfma(az[m], bq[m], acc);
    if (us == 0) {
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int gl = t0 + 4 * rb + x;
        if (gl < ng) cz_s[gl * 4 + hs] = acc[x] * p.scale2;
      }
    }
  }
  // query times the factor that undoes the field position of this lane's channels
  // (1 bit: 2^(lane%4), times 2^4 in odd 32-channel blocks; 2 bit: 4^(lane%4); 4 bit: 16^(lane%2))
  float qf[4][2];
  {
    const int shift = BITS == 1 ? lane % 4 + 4 * ((lane / 16) % 2) : BITS == 2 ? 2 * (lane % 4) : 4 * (lane % 2);
    const float comp = (float)(1 << kEK) / (float)(1 << shift);
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      const half2_t qq = as_half2(q2[hh]);
      qf[hh][0] = hh < G ? (float)qq[0] * comp : 0.f;
      qf[hh][1] = hh < G ? (float)qq[1] * comp : 0.f;
    }
  }
  TKV_PH();  // 1 this wave's set-up work done
  __syncthreads();  // cz table, tail slots, query copy and group counter are in place
  TKV_PH();  // 2 set-up done

  if (has_tail && wave < kTailWaves && wave * 32 < n - nq)
    tail_wave(p, tail_s[wave], q_h, bh, nq, n, p.residual + GRP, wave, lane);
  TKV_PH();  // 3 tail done

  // codes carry 2^-24, query side 2^kEK, so S = acc * 2^(24-kEK)
  const float K1 = p.scale2 * (float)(1 << (24 - kEK));

  floatx4 acc_o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc_o[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  floatx4 acc_z = {0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY;

  // A operand of the z_v / denominator MFMA: rows 0..NU-1 hold z_v[u = row] (loaded per group)
  // times the constant that undoes the weight-side scaling, row 4 holds that constant
  // alone (denominator), the other rows are zero.  Built branch-free as load * zmul + zadd.
  const int zrow = slot;                          // as A operand this lane holds row `slot`
  const int zrow_ld = zrow < NU ? zrow : NU - 1;  // other rows load a valid row and multiply it by 0
  half2_t zmul[4], zadd[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    // element k = 2j + e of this lane carries 2^-kEP * (2^j | 4^j | 16^(j%2))
    const int fs = BITS == 1 ? j : BITS == 2 ? 2 * j : 4 * (j % 2);
    const float w = (float)(1 << fs) / (float)(1 << kEP);
    const _Float16 wm = (_Float16)(zrow < NU ? w : 0.f), wa = (_Float16)(zrow == 4 ? w : 0.f);
    zmul[j] = half2_t{wm, wm};
    zadd[j] = half2_t{wa, wa};
  }
  // exponent offsets that put 2^kEP / (2^j | 4^j | 16^(j%2)) into the weights; value i of the
  // lane (tile tau = i/4, row x = i%4) is element kappa = 4 tau + x, register j = kappa/2
  float off[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int j = i / 2;
    off[i] = BITS == 1 ? (float)(kEP - j) : BITS == 2 ? (float)(kEP - 2 * j) : (float)(kEP - 4 * (j % 2));
  }

  // Next group index from the workgroup's LDS counter.  Written as inline assembly: the
  // compiler orders every LDS atomic it knows of behind all outstanding direct-to-LDS
  // loads (vmcnt(0)), which would drain the prefetch ring at every step.
  const uint32_t next_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)&s_next;
  auto grab = [&]() -> int {
    int v = 0;
    if (lane == 0) {
      const int one = 1;
      asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(next_addr), "v"(one) : "memory");
    }
    return __builtin_amdgcn_readfirstlane(v);
  };

  // ---- pipeline stages of one group.  Every stage is split into its LDS reads and its
  // arithmetic, so that a step can issue the reads well ahead of their use (a wave issues in
  // order: a read that is waited for right away stalls it for the whole LDS latency).
  // K: scalers x query -> hi/lo operands in LDS
  auto read_ks = [&](uint32_t so) -> uint32_t {
    return *reinterpret_cast<const uint32_t*>(smem + so + C::kCode + lane4);
  };
  auto stage_k = [&](uint32_t ks2) {
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      const uint32_t hi = mix_hi_pair(qf[hh][0], qf[hh][1], ks2);  // products are exact in float32
      bk_s[0][hh][lane] = hi;
      bk_s[1][hh][lane] = mix_lo_pair(qf[hh][0], qf[hh][1], ks2, hi);
    }
  };
  // QK: partial logits of the group's 32 tokens (two 16-token tiles); even column groups
  // read the hi rows of the query-side operand, odd ones the lo rows
  const uint32_t* bk_row = &bk_s[us & 1][hs][4 * rb];
  struct QkIn {
    uint32_t kw[C::kCodeWords];
    uintx4 bk[4];
  };
  auto read_codes = [&](const unsigned char* s, uint32_t (&cw)[C::kCodeWords]) {
    if (BITS == 1) {
      cw[0] = *reinterpret_cast<const uint32_t*>(s + lane4);
      cw[1] = *reinterpret_cast<const uint32_t*>(s + 256 + lane4);
    } else {
#pragma unroll
      for (int x = 0; x < BITS / 2; ++x) {
        const uintx4 t = *reinterpret_cast<const uintx4*>(s + 1024 * x + lane16);
#pragma unroll
        for (int y = 0; y < 4; ++y) cw[4 * x + y] = t[y];
      }
    }
  };
  auto read_qk = [&](uint32_t so, QkIn& in) {
    read_codes(smem + so, in.kw);
#pragma unroll
    for (int m = 0; m < 4; ++m) in.bk[m] = *reinterpret_cast<const uintx4*>(bk_row + 16 * m);
  };
  auto stage_qk = [&](const QkIn& in, floatx4 (&acc_s)[2]) {
    acc_s[0] = floatx4{0.f, 0.f, 0.f, 0.f};
    acc_s[1] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (BITS == 1) {
#pragma unroll
      for (int tau = 0; tau < 2; ++tau) {
        uintx4 a[4];
        extract1(in.kw[tau], a);
#pragma unroll
        for (int m = 0; m < 4; ++m) acc_s[tau] = mfma(a[m], in.bk[m], acc_s[tau]);
      }
      return;
    }
#pragma unroll
    for (int m2 = 0; m2 < 2; ++m2) {  // pairs of MFMA steps m = 2*m2, 2*m2+1
#pragma unroll
      for (int tau = 0; tau < 2; ++tau) {
        uintx4 a[2];
        if (BITS == 2) {
          extract2(in.kw[(2 * tau + m2) % C::kCodeWords], a[0], a[1]);
        } else {
          extract4(in.kw[(4 * tau + 2 * m2) % C::kCodeWords], a[0]);
          extract4(in.kw[(4 * tau + 2 * m2 + 1) % C::kCodeWords], a[1]);
        }
#pragma unroll
        for (int y = 0; y < 2; ++y) acc_s[tau] = mfma(a[y], in.bk[2 * m2 + y], acc_s[tau]);
      }
    }
  };
  // weights and weight-side operands
  struct PvIn {
    uintx4 sv, zv;
    uint32_t vw[C::kCodeWords];
    float cz;
  };
  auto read_pv = [&](uint32_t so, int gc, PvIn& in) {
    const unsigned char* s = smem + so;
    in.sv = *reinterpret_cast<const uintx4*>(s + C::oVs + ((us / GS) * TKV_BLK + 8 * rb) * 2);
    in.zv = *reinterpret_cast<const uintx4*>(s + C::oVz + (zrow_ld * TKV_BLK + 8 * rb) * 2);
    read_codes(s, in.vw);
    in.cz = cz_s[(gc - blk0) * 4 + hs];
  };
  struct POps {
    uintx4 b2, bp, a_zv;
  };
  // The weights 2^(x - m_run) go to the matrix cores as fp16, so m_run (a per-head reference,
  // not necessarily the running maximum) only has to keep them below 2^kHeadroomLog2: that
  // is checked on the weights themselves (an integer maximum of their bit patterns), and
  // only a failed check (rare after the first groups) pays for the exact maximum, the
  // accumulator rescale and a second pass.
  auto stage_soft = [&](const PvIn& in, const floatx4 (&acc_s)[2], POps& o) {
    const float cz = in.cz;
    float xs[8];  // hi + lo partial sums: every lane of a head ends up with the full logit
#pragma unroll
    for (int x = 0; x < 8; ++x) xs[x] = ror4_add(acc_s[x / 4][x % 4]);
    float pw[8];
    auto weights = [&]() {
      const float czm = cz - m_run;
#pragma unroll
      for (int x = 0; x < 8; ++x) pw[x] = __builtin_amdgcn_exp2f(__builtin_fmaf(xs[x], K1, czm + off[x]));
    };
    weights();
    {
      // bit patterns of non-negative floats (and of inf / NaN) order like integers
      uint32_t mm = 0u;
#pragma unroll
      for (int x = 0; x < 8; ++x) mm = max(mm, __builtin_bit_cast(uint32_t, pw[x]));
      constexpr uint32_t kLimit = (uint32_t)(127 + kEP + kHeadroomLog2) << 23;  // 2^(kEP + headroom)
      if (__builtin_amdgcn_ballot_w64(mm >= kLimit) != 0ull) {
        const float mx = fmaxf(fmaxf(fmaxf(xs[0], xs[1]), fmaxf(xs[2], xs[3])), fmaxf(fmaxf(xs[4], xs[5]), fmaxf(xs[6], xs[7])));
        float mn = __builtin_fmaf(mx, K1, cz);  // largest logit among this lane's 8 tokens
        mn = fmaxf(mn, __shfl_xor(mn, 4, 64));
        mn = fmaxf(mn, __shfl_xor(mn, 8, 64));
        mn = fmaxf(mn, __shfl_xor(mn, 16, 64));
        mn = fmaxf(mn, __shfl_xor(mn, 32, 64));
        // New reference: kRefBelowMax under the head's largest logit (never lower than before).
        // The largest weight is then 2^kRefBelowMax and the many small ones, which carry most of
        // the mass in a long context, sit that much further inside fp16's normal range.
        mn = fmaxf(m_run, mn - (float)kRefBelowMax);
        const float alpha = exp2f(m_run - mn);  // 0 on the first group
#pragma unroll
        for (int i = 0; i < 8; ++i) acc_o[i] *= alpha;
        acc_z *= alpha;
        m_run = mn;
        weights();
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float2_t w2 = {pw[2 * j], pw[2 * j + 1]};
      o.bp[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(w2, half2_t));
      // weight x scaler: one rounding of the exact product of two fp16 numbers
      const uint32_t bpj = o.bp[j], svj = in.sv[j], zvj = in.zv[j];
      o.b2[j] = __builtin_bit_cast(uint32_t, as_half2(bpj) * as_half2(svj));
      const half2_t t = __builtin_elementwise_fma(as_half2(zvj), zmul[j], zadd[j]);
      o.a_zv[j] = __builtin_bit_cast(uint32_t, t);
    }
  };
  // P.V: 8 blocks of 16 channels + the z_v / denominator MFMA
  auto stage_pv = [&](const PvIn& in, const POps& o) {
    acc_z = mfma(o.a_zv, o.bp, acc_z);
    if (BITS == 1) {
#pragma unroll
      for (int wd = 0; wd < 2; ++wd) {
        uintx4 a[4];
        extract1(in.vw[wd], a);
#pragma unroll
        for (int y = 0; y < 4; ++y) acc_o[4 * wd + y] = mfma(a[y], o.b2, acc_o[4 * wd + y]);
      }
      return;
    }
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) {
      uintx4 a[2];
      if (BITS == 2) {
        extract2(in.vw[wd % C::kCodeWords], a[0], a[1]);
      } else {
        extract4(in.vw[((wd / 2) * 4 + 2 * (wd % 2)) % C::kCodeWords], a[0]);
        extract4(in.vw[((wd / 2) * 4 + 2 * (wd % 2) + 1) % C::kCodeWords], a[1]);
      }
#pragma unroll
      for (int y = 0; y < 2; ++y) acc_o[2 * wd + y] = mfma(a[y], o.b2, acc_o[2 * wd + y]);
    }
  };
#define TKV_WAIT_VMCNT(N) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory")
  constexpr int L = C::kKLoads + C::kVLoads;  // load instructions issued per pipeline step

  // ---- software pipeline over this wave's groups g[0], g[1], ...  Step i computes the
  // logits of group i+1, the weights and P.V of group i and the query-side operand of
  // group i+2, while the K part of group i+3 and the V part of group i+2 are in flight.
  if (active) {
    floatx4 acc_a[2], acc_b[2];
    TKV_WAIT_VMCNT(2 * C::kKLoads + C::kVLoads);  // K0, V0 landed
    stage_k(read_ks(kl));
    {
      QkIn qi;
      read_qk(kl, qi);
      stage_qk(qi, acc_a);
    }
    TKV_WAIT_VMCNT(L);  // + K1
    stage_k(read_ks(kq));
    // One step is one straight-line block; groups past the chunk are clamped copies whose
    // results are dropped by leaving the loop.  gc = group i (valid), gn3 / gv2 = groups
    // whose K / V part is fetched now.  LDS reads go out one stage ahead of their use.
    auto step = [&](int gc, int gn3, int gv2, floatx4 (&acc_c)[2], floatx4 (&acc_n)[2]) {
      QkIn qi;
      read_qk(kq, qi);  // K(i+1) landed during the previous step
      __builtin_amdgcn_sched_barrier(0);
      load_kpart(kl, gn3);
      load_vpart(vl, gv2);
      TKV_WAIT_VMCNT(2 * L);  // K(i+1), V(i) landed
      PvIn pi;
      read_pv(vp, gc, pi);
      __builtin_amdgcn_sched_barrier(0);
      stage_qk(qi, acc_n);
      POps po;
      stage_soft(pi, acc_c, po);
      TKV_WAIT_VMCNT(L + C::kVLoads);  // + K(i+2)
      const uint32_t ks2 = read_ks(kk);
      __builtin_amdgcn_sched_barrier(0);
      stage_pv(pi, po);
      stage_k(ks2);
      uint32_t t = kq;
      kq = kk, kk = kl, kl = t;
      t = vp;
      vp = vn, vn = vl, vl = t;
    };
    int gc = g0;
    for (;;) {
      const int g3 = grab();
      step(gc, g3, g2, acc_a, acc_b);
      if (g1 >= blk1) break;
      const int g4 = grab();
      step(g1, g4, g3, acc_b, acc_a);
      if (g2 >= blk1) break;
      gc = g2;  // rotate: group i+2 becomes the current one
      g1 = g3;
      g2 = g4;
    }
  }
#undef TKV_WAIT_VMCNT
  TKV_PH();  // 4 this wave's groups done
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no direct-to-LDS load may land after the ring is reused

  // ---- per-wave results -> LDS, each wave into its own (now idle) ring, so no wave waits for
  // another before writing.  acc_z rows: lanes 0..15 (rb 0) hold rows 0..3 = z-terms for
  // u = row; lanes 16..31 register 0 hold row 4 = denominator.
  auto merge_of = [&](int w) -> MergeWave& { return *reinterpret_cast<MergeWave*>(smem + C::oRing + w * C::kWaveRing); };
  MergeWave& mw = merge_of(wave);
  if (rb == 0) {
#pragma unroll
    for (int x = 0; x < 4; ++x)
      if (x == us / GS) mw.z[hs][us] = acc_z[x];
    if (us == 0) mw.m[hs] = m_run;
  }
  if (rb == 1 && us == 0) mw.l[hs] = acc_z[0];
  {
    // written by lanes of this same wave just above: a wave's LDS operations execute in order
    const float zt = mw.z[hs][us];
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
      // 1 bit: the codes of odd 16-channel blocks sit four mantissa bits higher
      const float unscale = (float)(1 << (24 - kEP - (BITS == 1 && cb % 2 ? 4 : 0)));
      if (cb / 2 == us) {
#pragma unroll
        for (int x = 0; x < 4; ++x) mw.o[hs][16 * cb + 4 * rb + x] = __builtin_fmaf(acc_o[cb][x], unscale, zt);
      }
    }
  }
  __syncthreads();
  TKV_PH();  // 5 all waves done, results in LDS
  // merge weights of the W wave entries and the tail entries: every wave works them out for
  // itself (lane = (entry, head)) into arrays of its own, which spares the workgroup a barrier
  constexpr int NE = W + kTailWaves;
  __shared__ float s_w_all[W][NE][4];
  __shared__ float s_ml_all[W][2][4];
  static_assert(NE <= 16, "one wave covers all (entry, head) pairs");
  float(*s_w)[4] = s_w_all[wave];
  float(*s_ml)[4] = s_ml_all[wave];
  {
    const int e = lane / 4, hh = lane % 4;
    float me = -INFINITY, le = 0.f;
    if (e < W) {
      me = merge_of(e).m[hh];
      le = merge_of(e).l[hh];
    } else if (e < NE) {
      me = tail_s[e - W].m[hh];
      le = tail_s[e - W].l[hh];
    }
    float M = me;
    for (int m = 4; m <= 32; m <<= 1) M = fmaxf(M, __shfl_xor(M, m, 64));
    const float wgt = me == -INFINITY ? 0.f : exp2f(me - M);
    float Lsum = le * wgt;
    for (int m = 4; m <= 32; m <<= 1) Lsum += __shfl_xor(Lsum, m, 64);
    if (e < NE) s_w[e][hh] = wgt;
    if (e == 0) {
      s_ml[0][hh] = M;
      s_ml[1][hh] = Lsum;
    }
  }
  for (int i = tid; i < G * TKV_D; i += C::kThreads) {
    const int hh = i / TKV_D, c = i % TKV_D;
    float O = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) O = __builtin_fmaf(merge_of(w).o[hh][c], s_w[w][hh], O);
#pragma unroll
    for (int w = 0; w < kTailWaves; ++w) {  // unused tail slots hold no data, only a zero weight
      const float wgt = s_w[W + w][hh];
      O = __builtin_fmaf(wgt != 0.f ? tail_s[w].o[hh][c] : 0.f, wgt, O);
    }
    float* dst = p.parts + (((size_t)chunk_base * p.hq + ((size_t)qh0 + hh) * n_chunks) + chunk) * TKV_PART_STRIDE;
    // device-scope stores: visible to the merging workgroup without a cache write-back
    __hip_atomic_store(dst + TKV_PART_O + c, O, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (c == 0) {
      __hip_atomic_store(dst, s_ml[0][hh], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(dst + 1, s_ml[1][hh], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- the last workgroup of this (sequence, KV head) to arrive merges all chunks.
  // Partials travel through device-scope (cache-bypassing) stores and loads, ordered by
  // waiting for the stores to complete before the arrival counter is bumped: a release /
  // acquire fence pair would write back and invalidate the whole L2 (tens of microseconds).
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  TKV_PH();  // 6 partial written
  __syncthreads();
  uint32_t* arrival = p.arrivals + (size_t)b * gridDim.y + blockIdx.y;
  if (tid == 0) s_flag = atomicAdd(arrival, 1u) == (uint32_t)(n_chunks - 1) ? 1u : 0u;
  __syncthreads();
  if (s_flag != 0u) {
    if (tid == 0) *arrival = 0u;
    const float* head0 = p.parts + ((size_t)chunk_base * p.hq + (size_t)qh0 * n_chunks) * TKV_PART_STRIDE;
    float* scratch = reinterpret_cast<float*>(smem + C::oRing);  // the waves' results have been consumed
    tkv::merge_chunks(head0, G, n_chunks, p.out + ((size_t)b * p.hq + (size_t)qh0) * TKV_D, scratch, tid, C::kThreads);
  }
  TKV_PH();  // 7 end
#ifdef TKV_PHASE
  if (p.prof && lane == 0) {
    long long* dst = p.prof + ((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * W + wave) * 8;
    for (int i = 0; i < 8; ++i) dst[i] = ph[i];
  }
#endif
}

template <int BITS, int GS, int W>
int32_t launch_variant(const MfmaParams& p, dim3 grid, hipStream_t s) {
  using C = Cfg<BITS, GS, W>;
  // more than 64 KiB of dynamic LDS needs an opt-in, once per kernel
  static const bool lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&quant_attn_mfma_kernel<BITS, GS, W>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes) == hipSuccess;
  if (!lds_ok) return TKV_E_HIP;
  TKV_LAUNCH((quant_attn_mfma_kernel<BITS, GS, W>), grid, C::kThreads, C::kLdsBytes, s, p);
  return TKV_OK;
}

}  // namespace

namespace tkv {
#ifdef TKV_PHASE
void* g_mfma_prof = nullptr;
#endif

// Chunks per (sequence, KV head): about `target_blocks` workgroups in total (one per
// compute unit), at least one 32-token block per wave, and no more blocks per chunk than
// the zero-point table of a workgroup holds.
int32_t launch_quant_attn_mfma(const tkv_quant_desc* d, const tkv_quant_cache* c, const __half* q, __half* out,
                               float scale2, float* parts, size_t parts_floats, uint32_t* arrivals, int target_blocks,
                               int max_groups, int max_tail, const TkvSeqLens& lens, const QuantNewTokens* fresh,
                               hipStream_t s) {
  if (d->head_dim != TKV_D) return TKV_E_UNSUPPORTED;
  // built: the benchmark's settings (2 and 4 bit, groups of 32) and the paper's (1 and 2 bit, groups of 64)
  const int variant = d->bits * 100 + d->group_size;
  if (variant != 232 && variant != 432 && variant != 164 && variant != 264) return TKV_E_UNSUPPORTED;
  const int waves = d->bits == 4 ? 8 : 12;
  // Chunks per KV head over the whole batch: about target_blocks workgroups in all, shared out
  // among the sequences in proportion to their work (32-token blocks, a 32-token piece of the
  // fp16 tail counting as two), so that every workgroup sweeps about the same number of blocks
  // whatever the mix of lengths.  Per sequence: at least one block per wave, at most 64 chunks
  // (unless the tuning hook asks for more workgroups than that gives), no more blocks per chunk
  // than the zero-point table of a workgroup holds.
  (void)max_groups;
  (void)max_tail;
  MfmaParams p;
  const int split = (d->n_q_heads / d->n_kv_heads + 3) / 4;  // workgroups per KV head and chunk: 4 query heads each
  const int heads = d->n_kv_heads * split;
  int per_head = (target_blocks + heads - 1) / heads;
  if (per_head < d->batch) per_head = d->batch;
  const int chunk_cap = target_blocks > 64 * d->batch * heads ? TKV_MAX_CHUNKS : 64;
  long long total_work = 0;
  int work[TKV_MAX_BATCH];
  for (int b = 0; b < d->batch; ++b) {
    const int n = lens.n[b];
    const int g = tkv::n_quantized(n, d->residual, d->group_size) / TKV_BLK;
    work[b] = g + 2 * ((n - g * TKV_BLK + 31) / 32);
    total_work += work[b];
  }
  int total_chunks = 0;
  for (int b = 0; b < d->batch; ++b) {
    int nc = total_work > 0 ? (int)(((long long)per_head * work[b] + total_work / 2) / total_work) : 1;
    const int c_work = (work[b] + waves - 1) / waves;
    if (nc > c_work) nc = c_work;
    if (nc > chunk_cap) nc = chunk_cap;
    if (nc < 1) nc = 1;
    if ((work[b] + nc - 1) / nc > kMaxGpc) nc = (work[b] + kMaxGpc - 1) / kMaxGpc;
    if (nc > TKV_MAX_CHUNKS) return TKV_E_UNSUPPORTED;
    p.chunks.n[b] = nc;
    total_chunks += nc;
  }
  // Rounding may leave a few chunks too many (a second round of workgroups for a handful of
  // them) or too few (idle compute units): take them from the sequences whose chunks are the
  // lightest, give them to those whose chunks are the heaviest.
  while (total_chunks > per_head) {
    int pick = -1;
    for (int b = 0; b < d->batch; ++b) {
      const int nc = p.chunks.n[b];
      if (nc <= 1 || (work[b] + nc - 2) / (nc - 1) > kMaxGpc) continue;
      if (pick < 0 || (long long)work[b] * (p.chunks.n[pick] - 1) < (long long)work[pick] * (nc - 1)) pick = b;
    }
    if (pick < 0) break;
    --p.chunks.n[pick];
    --total_chunks;
  }
  while (total_chunks < per_head) {
    int pick = -1;
    for (int b = 0; b < d->batch; ++b) {
      const int nc = p.chunks.n[b];
      if (nc >= chunk_cap || nc >= (work[b] + waves - 1) / waves) continue;
      if (pick < 0 || (long long)work[b] * p.chunks.n[pick] > (long long)work[pick] * nc) pick = b;
    }
    if (pick < 0) break;
    ++p.chunks.n[pick];
    ++total_chunks;
  }
  if ((size_t)total_chunks * d->n_q_heads * TKV_PART_STRIDE > parts_floats) return TKV_E_WORKSPACE;
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
  p.batch = d->batch;
#ifdef TKV_PHASE
  p.prof = (long long*)g_mfma_prof;
#endif
  p.lens = lens;
  p.k_new = nullptr;
  if (fresh != nullptr) {
    p.k_new = fresh->k_new;
    p.v_new = fresh->v_new;
    p.n_stride = fresh->n_stride;
    p.n_add = fresh->n_add;
  }
  const dim3 grid(total_chunks, heads, 1);
  switch (variant) {
    case 232: return launch_variant<2, 1, 12>(p, grid, s);
    case 432: return launch_variant<4, 1, 8>(p, grid, s);
    case 164: return launch_variant<1, 2, 12>(p, grid, s);
    case 264: return launch_variant<2, 2, 12>(p, grid, s);
  }
  return TKV_E_UNSUPPORTED;
}

}  // namespace tkv

#ifdef TKV_PHASE
// profiling builds (-DTKV_PHASE): device buffer that receives [workgroup][wave][8] wall-clock stamps
extern "C" void tkv_debug_set_dump(void* ptr) { tkv::g_mfma_prof = ptr; }
#endif
