// Offline identification (Sec. 4.1): dense preference score of a layer, Eq. 6-8, and the
// classification of Eq. 9.
//
// Per (sequence, KV head) the attention logits of the R = G * n_q most recent query rows
// against all n keys are a dense contraction (v_mfma_f32_16x16x32_f16); what Eq. 7 needs of a
// row is not the index set of its top_k entries but their softmax mass, which ties do not
// change.  Logits are never written to memory: they are computed twice.
//
//   pass 1  logits -> "block maxima": every (row, lane slot of a wave) keeps the maximum of
//           the <= 32 logits it sees in a round of 8 key chunks.  The blocks of a row are
//           disjoint, so the top_k-th largest block maximum L is a lower bound of the row's
//           top_k-th largest logit T (top_k distinct logits are >= L), and because a block
//           holds few keys, spread over the sequence, it is a tight one: with keys in random
//           order about 1.15 top_k logits reach L.  At most 32 (top_k - 1) logits can lie
//           above L whatever the data (each lies in a block whose maximum does).
//   bound   per row: L (radix select over the block maxima) and the row maximum m.
//   pass 2  the same logits again, bit for bit (same instructions on the same operands):
//           softmax denominator against m, the logits above L appended to the row's
//           candidate list (through per-workgroup lists in LDS), the logits equal to L counted.
//   final   per row: T = top_k-th largest candidate if there are top_k of them, else L (the
//           rest of the top_k entries are ties at L); mass of the top_k entries, summed in
//           64-bit fixed point so that the result does not depend on the order in which
//           candidates were appended; Eq. 8 per head in row order.
//
// Shape of the two passes: a workgroup of 16 waves owns 256 rows (4 waves per SIMD: query
// group g = wave % 8 holds its 32 rows as MFMA B operands in registers) and every P-th chunk
// of 128 keys; a chunk is staged once in LDS (direct global -> LDS loads, three or four buffers deep, one
// barrier per chunk) and read by all waves as A operands; wave (g, s) takes key tiles s, s + 2, s + 4, s + 6 of the
// chunk, 8 MFMAs per tile.  D layout: a lane holds 4 keys x 1 query, so a row's constants (L, m) and
// its partial denominator are per-lane scalars.
#include <algorithm>
#include <type_traits>

#include "tkv_common.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 1024;
constexpr int kSlabRows = 256;       // rows per workgroup
constexpr int kChunk = 128;          // keys per staged chunk
constexpr int kChunkBytes = kChunk * 256;
constexpr int kRing1 = 4;            // chunk buffers in LDS: pass 1 (bound by the key stream)
constexpr int kRing2 = 3;            // pass 2 (bound by its arithmetic; the candidate lists need the room)
constexpr int kQT = 2;               // query tiles (16 rows each) per wave
constexpr int kSubLanes = 2;         // waves that share the key tiles of a chunk for the same rows
constexpr int kGroups = 16 / kSubLanes;            // query groups of a workgroup
constexpr int kTilesPerWave = kChunk / 16 / kSubLanes;  // key tiles of a chunk per wave
constexpr int kRound = 8;            // chunks per block-maximum round: 8 chunks x 4 tiles = 32 keys per block
constexpr int kBlockKeys = kRound * kTilesPerWave;
constexpr int kBlocksPerRound = kSubLanes * 16;  // per row and workgroup: key sub-lanes x 16 lane slots
static_assert(kGroups * kQT * 16 == kSlabRows, "rows of a workgroup");
constexpr int kListCap = 56;         // candidates per row kept in LDS by a workgroup; further ones go straight to memory
constexpr int kPass1Lds = kRing1 * kChunkBytes;
constexpr int kPass2Lds = kRing2 * kChunkBytes + kSlabRows * kListCap * 4 + 2 * kSlabRows * 4;
static_assert(kPass2Lds <= 160 * 1024, "LDS of pass 2");

struct PrefParams {
  const __half* q_last;  // [B][n_q][Hq][128]
  const __half* k;       // [B][n][Hkv][128]
  float* blkmax;         // [Hkv][R][nblk]
  float* bound;          // [Hkv][R][2]: L, row maximum (raw dot products)
  float* den;            // [Hkv][R][P]: partial softmax denominators
  float* cand;           // [Hkv][R][cand_cap]: logits above L, in no particular order
  uint32_t* cursor;      // [Hkv][R][2]: candidates stored, logits equal to L; zero between calls
  float* row_p;          // [Hkv][R]
  float* p_out;          // [B][Hq]
  float scale2;          // sm_scale * log2(e)
  int32_t hq, hkv, n_q, n, b, top_k;
  int32_t P;             // workgroups per (KV head, slab): workgroup r owns chunks r, r + P, ...
  int32_t rounds;        // block-maximum rounds of a workgroup
  int32_t nblk;          // P * rounds * kBlocksPerRound
  int32_t cand_cap;
};

__device__ inline uint32_t float_key(float s) {
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

__device__ inline void lds_load16(const void* g, void* l) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}
#define TKV_WAIT_VMCNT(N) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory")

// LDS counter += 1, old value back.  In assembly: the compiler orders every LDS atomic it
// knows behind all outstanding direct-to-LDS loads, which would stall the load ring.
__device__ inline uint32_t lds_inc(uint32_t* addr) {
  uint32_t old;
  const uint32_t one = 1u;
  const uint32_t a = (uint32_t)(uintptr_t)addr;
  asm volatile("ds_add_rtn_u32 %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=v"(old) : "v"(a), "v"(one) : "memory");
  return old;
}

// max(a, b) as the median of (a, b, +inf): one instruction, where fmaxf costs three (it quiets
// NaNs in both operands first; no NaN is expected here, and none could be selected)
__device__ inline float max_f32(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, INFINITY); }

// PASS 1: block maxima.  PASS 2: denominators and candidates.
//
// Key chunks travel global -> LDS directly (no registers), into a ring of buffers: while chunk i
// is computed on, the next two (pass 2) or three (pass 1) are in flight.  A load instruction of a wave fills 1 KiB
// of LDS in lane order, i.e. 4 key rows of 256 bytes; the lanes pick their 16-byte pieces so
// that piece c of row r lands at slot (c + r) mod 16 of its row: the A-operand reads (16 rows,
// same piece) then touch 16 different slots and are free of bank conflicts.
template <int PASS>
__global__ __launch_bounds__(kThreads) void pref_pass_kernel(PrefParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int kRing = PASS == 1 ? kRing1 : kRing2;
  float* llist = reinterpret_cast<float*>(smem + kRing * kChunkBytes);                                // [256][kListCap]
  uint32_t* lcnt = reinterpret_cast<uint32_t*>(smem + kRing * kChunkBytes + kSlabRows * kListCap * 4);  // [256]
  uint32_t* leq = lcnt + kSlabRows;                                                                    // [256]
  const int tid = threadIdx.x, lane = tid % 64, wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int g = wave % kGroups, s = wave / kGroups;
  const int col = lane % 16, kb = lane / 16;
  const int r_wg = blockIdx.x, h = blockIdx.y, slab = blockIdx.z;
  const int G = p.hq / p.hkv, R = G * p.n_q;
  const int row0 = slab * kSlabRows + g * (16 * kQT);  // first row of this wave
  const int nqt = max(0, min(kQT, (R - row0) / 16));   // query tiles of this wave (R is a multiple of 16)
  const int n_chunks = (p.n + kChunk - 1) / kChunk;
  const int my_chunks = r_wg < n_chunks ? (n_chunks - r_wg + p.P - 1) / p.P : 0;

  // B operands: this wave's query rows (row = query head of the group * n_q + position)
  uintx4 bq[kQT][4];
#pragma unroll
  for (int qt = 0; qt < kQT; ++qt) {
    const int r = min(row0 + 16 * qt + col, R - 1), j = r / p.n_q, i = r % p.n_q;
    const __half* qrow = p.q_last + (((size_t)p.b * p.n_q + i) * p.hq + (size_t)h * G + j) * TKV_D;
#pragma unroll
    for (int m = 0; m < 4; ++m) bq[qt][m] = *reinterpret_cast<const uintx4*>(qrow + 32 * m + 8 * kb);
  }
  float L[kQT], mrow[kQT], den[kQT];
  if (PASS == 2) {
    for (int x = tid; x < 2 * kSlabRows; x += kThreads) lcnt[x] = 0;
#pragma unroll
    for (int qt = 0; qt < kQT; ++qt) {
      const int r = min(row0 + 16 * qt + col, R - 1);
      const float2 lm = *reinterpret_cast<const float2*>(p.bound + ((size_t)h * R + r) * 2);
      L[qt] = lm.x, mrow[qt] = -lm.y * p.scale2, den[qt] = 0.f;  // (minus the row maximum, log2 units)
    }
  }
  float bm[kQT][4];
#pragma unroll
  for (int qt = 0; qt < kQT; ++qt)
#pragma unroll
    for (int x = 0; x < 4; ++x) bm[qt][x] = -INFINITY;

  // this wave brings rows 8 wave .. 8 wave + 7 of every chunk: two load instructions
  const int lrow = lane / 16, lslot = lane % 16;
  auto load_chunk = [&](int c, int buf) {
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int r = 8 * wave + 4 * y + lrow;               // row of the chunk
      const int key = min(c * kChunk + r, p.n - 1);         // keys past the end re-read the last one and are masked below
      const int piece = (lslot - r) & 15;
      const __half* src = p.k + (((size_t)p.b * p.n + key) * p.hkv + h) * TKV_D + 8 * piece;
      lds_load16(src, smem + buf * kChunkBytes + (8 * wave + 4 * y) * 256);
    }
  };

  // one key tile of the chunk in buffer `base` against this wave's rows
  auto tile_step = [&](const unsigned char* base, int c, int tile, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;  // all four query tiles present, no key past the end
    const int key0 = c * kChunk + tile * 16;
    floatx4 acc[kQT];
#pragma unroll
    for (int qt = 0; qt < kQT; ++qt) acc[qt] = floatx4{0.f, 0.f, 0.f, 0.f};
    const unsigned char* arow = base + (tile * 16 + col) * 256;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uintx4 a = *reinterpret_cast<const uintx4*>(arow + ((4 * m + kb + col) & 15) * 16);
#pragma unroll
      for (int qt = 0; qt < kQT; ++qt)
        if (FULL || qt < nqt)
          acc[qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a),
                                                           __builtin_bit_cast(half8, bq[qt][m]), acc[qt], 0, 0, 0);
    }
    // this lane: keys key0 + 4 kb + x of the query row (row0 + 16 qt + col); logits stay in units
    // of the raw dot product (sm_scale > 0 keeps their order)
    if (PASS == 1) {
#pragma unroll
      for (int qt = 0; qt < kQT; ++qt) {
        if (!FULL && qt >= nqt) continue;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const bool valid = FULL || key0 + 4 * kb + x < p.n;
          bm[qt][x] = max_f32(bm[qt][x], valid ? acc[qt][x] : -INFINITY);
        }
      }
      return;
    }
    // PASS 2.  About one logit in a hundred reaches L: a wave sees a few per tile, a lane almost
    // never more than one.  One test per lane and tile (is its largest logit of a row at or above
    // the row's L?), and only the lanes that pass look at their logits one by one.
    bool any = false;
#pragma unroll
    for (int qt = 0; qt < kQT; ++qt) {
      if (!FULL && qt >= nqt) continue;
      float mx = -INFINITY;
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const float v = acc[qt][x];
        const bool valid = FULL || key0 + 4 * kb + x < p.n;
        den[qt] += valid ? __builtin_amdgcn_exp2f(fmaf(v, p.scale2, mrow[qt])) : 0.f;
        mx = max_f32(mx, valid ? v : -INFINITY);
      }
      any = any || mx >= L[qt];
    }
    if (__builtin_amdgcn_ballot_w64(any) != 0) {
      if (any) {
        uint32_t hits = 0;
#pragma unroll
        for (int qt = 0; qt < kQT; ++qt) {
          if (!FULL && qt >= nqt) continue;
#pragma unroll
          for (int x = 0; x < 4; ++x)
            hits |= ((FULL || key0 + 4 * kb + x < p.n) && acc[qt][x] >= L[qt]) ? 1u << (4 * qt + x) : 0u;
        }
        while (hits != 0) {
          const int idx = __builtin_ctz(hits);
          hits &= hits - 1;
          float v = acc[0][0];
#pragma unroll
          for (int j = 1; j < 4 * kQT; ++j) v = idx == j ? acc[j / 4][j % 4] : v;
          const int qt = idx >> 2;
          float lq = L[0];
#pragma unroll
          for (int j = 1; j < kQT; ++j) lq = qt == j ? L[j] : lq;
          const int rl = g * (16 * kQT) + 16 * qt + col;
          if (v > lq) {
            const uint32_t slot = lds_inc(&lcnt[rl]);
            if (slot < (uint32_t)kListCap) {
              llist[rl * kListCap + slot] = v;
            } else {
              const size_t gr = (size_t)h * R + slab * kSlabRows + rl;
              const uint32_t gs = atomicAdd(&p.cursor[gr * 2], 1u);
              if (gs < (uint32_t)p.cand_cap) p.cand[gr * p.cand_cap + gs] = v;
            }
          } else {
            lds_inc(&leq[rl]);
          }
        }
      }
    }
  };

#pragma unroll
  for (int a = 0; a < kRing - 1; ++a)
    if (a < my_chunks) load_chunk(r_wg + a * p.P, a);
  for (int i = 0; i < my_chunks; ++i) {
    const int c = r_wg + i * p.P;
    // this wave's rows of chunk i have landed: loads retire in order, and those of the chunks
    // after it (two instructions each) may still be out
    const int ahead = min(kRing - 2, my_chunks - 1 - i);
    if (ahead >= 2) TKV_WAIT_VMCNT(4); else if (ahead == 1) TKV_WAIT_VMCNT(2); else TKV_WAIT_VMCNT(0);
    // everyone's rows of chunk i are there, and everyone is through with chunk i-1 (its operand
    // reads have returned).  A bare barrier: __syncthreads() would also wait for the loads in flight.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (i + kRing - 1 < my_chunks) load_chunk(c + (kRing - 1) * p.P, (i + kRing - 1) % kRing);
    const int buf = i % kRing;
    if (nqt > 0) {
      const unsigned char* base = smem + buf * kChunkBytes;
      const bool full = nqt == kQT && (c + 1) * kChunk <= p.n;
      if (full) {
#pragma unroll
        for (int tt = 0; tt < kTilesPerWave; ++tt) tile_step(base, c, s + kSubLanes * tt, std::true_type{});
      } else {
        for (int tt = 0; tt < kTilesPerWave; ++tt)
          if (c * kChunk + (s + kSubLanes * tt) * 16 < p.n)  // (wave-uniform)
            tile_step(base, c, s + kSubLanes * tt, std::false_type{});
      }
    }
    if (PASS == 1 && (i % kRound == kRound - 1 || i == my_chunks - 1)) {
      const int f = i / kRound;
#pragma unroll
      for (int qt = 0; qt < kQT; ++qt) {
        if (qt < nqt) {
          float* dst = p.blkmax + ((size_t)h * R + row0 + 16 * qt + col) * p.nblk +
                       ((size_t)(r_wg * p.rounds + f) * kSubLanes + s) * 16 + 4 * kb;
          *reinterpret_cast<float4*>(dst) = make_float4(bm[qt][0], bm[qt][1], bm[qt][2], bm[qt][3]);
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) bm[qt][x] = -INFINITY;
      }
    }
  }
  if (PASS == 1) {
    // rounds this workgroup has no chunks for: nothing was seen
    const int done = (my_chunks + kRound - 1) / kRound;
    for (int f = done; f < p.rounds; ++f)
#pragma unroll
      for (int qt = 0; qt < kQT; ++qt)
        if (qt < nqt) {
          float* dst = p.blkmax + ((size_t)h * R + row0 + 16 * qt + col) * p.nblk +
                       ((size_t)(r_wg * p.rounds + f) * kSubLanes + s) * 16 + 4 * kb;
          *reinterpret_cast<float4*>(dst) = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        }
    return;
  }
  // ---- pass 2 epilogue: denominators (fixed order: key lanes, then key sub-lanes), lists to memory
  __syncthreads();  // every wave is through with the chunk buffers: they now hold the partial denominators
  float* dsum = reinterpret_cast<float*>(smem);  // [sub-lanes][256 rows]
#pragma unroll
  for (int qt = 0; qt < kQT; ++qt) {
    float d = den[qt];
    d += __shfl_xor(d, 16, 64);
    d += __shfl_xor(d, 32, 64);
    if (kb == 0 && qt < nqt) dsum[s * kSlabRows + g * (16 * kQT) + 16 * qt + col] = d;
  }
  __syncthreads();
  const int rows_here = min(kSlabRows, R - slab * kSlabRows);
  if (tid < rows_here) {
    const size_t gr = (size_t)h * R + slab * kSlabRows + tid;
    float d = dsum[tid];
#pragma unroll
    for (int x = 1; x < kSubLanes; ++x) d += dsum[x * kSlabRows + tid];
    p.den[gr * p.P + r_wg] = d;
    const uint32_t eq = leq[tid];
    if (eq != 0) atomicAdd(&p.cursor[gr * 2 + 1], eq);
  }
  // a row's list: one quarter-wave of 16 lanes per row at a time
  for (int rl = tid / 16; rl < rows_here; rl += kThreads / 16) {
    const uint32_t cnt = min(lcnt[rl], (uint32_t)kListCap);
    if (cnt == 0) continue;
    const size_t gr = (size_t)h * R + slab * kSlabRows + rl;
    uint32_t base = 0;
    if (tid % 16 == 0) base = atomicAdd(&p.cursor[gr * 2], cnt);
    base = __shfl(base, lane & ~15, 64);
    for (uint32_t e = tid % 16; e < cnt; e += 16)
      if (base + e < (uint32_t)p.cand_cap) p.cand[gr * p.cand_cap + base + e] = llist[rl * kListCap + e];
  }
}

constexpr int kSelRegs = 16;  // values per thread that the selection kernels keep in registers

// The values of a row, as order-preserving keys: held in registers when there are at most
// 256 * kSelRegs of them (value e at thread e % 256), else streamed from memory every time.
struct RowKeys {
  const float* src;
  uint32_t count;
  bool cached;
  uint32_t reg[kSelRegs];
  __device__ void load(const float* s, uint32_t n) {
    src = s, count = n, cached = n <= 256u * kSelRegs;
    if (cached) {
#pragma unroll
      for (int j = 0; j < kSelRegs; ++j) {
        const uint32_t e = threadIdx.x + 256u * j;
        reg[j] = e < n ? float_key(s[e]) : 0u;
      }
    }
  }
  template <typename F>
  __device__ void for_each(F f) const {
    if (cached) {
#pragma unroll
      for (int j = 0; j < kSelRegs; ++j)
        if (threadIdx.x + 256u * j < count) f(reg[j]);
    } else {
      for (uint32_t e = threadIdx.x; e < count; e += 256) f(float_key(src[e]));
    }
  }
};

// the rank-th largest (1 <= rank <= count) of a row's keys, by a workgroup of 256 threads:
// radix select, 8 bits per pass, over the bits below the keys' common prefix only (a row's
// keys lie close together: with digits taken from the top of the key, every LDS atomic of
// the first passes would hit the same few counters and be serialized).
// hist: 256 words of LDS, s_pick: 4 words.
__device__ inline uint32_t kth_largest_key(const RowKeys& keys, uint32_t rank, uint32_t* hist, uint32_t* s_pick) {
  const int tid = threadIdx.x;
  uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
  keys.for_each([&](uint32_t key) { kmin = min(kmin, key), kmax = max(kmax, key); });
  for (int d = 32; d >= 1; d >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, d, 64));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, d, 64));
  }
  if (tid == 0) s_pick[2] = 0xFFFFFFFFu, s_pick[3] = 0u;
  __syncthreads();
  if (tid % 64 == 0) atomicMin(&s_pick[2], kmin), atomicMax(&s_pick[3], kmax);
  __syncthreads();
  kmin = s_pick[2], kmax = s_pick[3];
  int bits_left = 32 - __builtin_clz((kmin ^ kmax) | 1u);  // bits that differ between some keys (at least 1)
  uint32_t prefix = bits_left == 32 ? 0u : (kmax >> bits_left) << bits_left;
  uint32_t remaining = rank;
  while (bits_left > 0) {
    const int w = min(8, bits_left), shift = bits_left - w;
    hist[tid] = 0;
    __syncthreads();
    const uint32_t hi_mask = bits_left == 32 ? 0u : (0xFFFFFFFFu << bits_left);
    const uint32_t dmask = (1u << w) - 1u;
    keys.for_each([&](uint32_t key) {
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & dmask], 1u);
    });
    __syncthreads();
    if (tid < 64) {
      // wave 0: suffix sums over the 256 bins, 4 bins per lane, highest digit first
      const int l = tid;
      uint32_t c[4], tot = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) c[j] = hist[255 - (4 * l + j)], tot += c[j];
      uint32_t incl = tot;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d, 64);
        if (l >= d) incl += o;
      }
      uint32_t run = incl - tot;  // entries in higher digits than this lane's
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (run < remaining && remaining <= run + c[j]) {
          s_pick[0] = 255 - (4 * l + j);
          s_pick[1] = remaining - run;
        }
        run += c[j];
      }
    }
    __syncthreads();
    prefix |= s_pick[0] << shift;
    remaining = s_pick[1];
    bits_left = shift;
    __syncthreads();
  }
  return prefix;
}

// One workgroup per row: L = the top_k-th largest block maximum (-inf if the row has fewer
// blocks than that), m = the row maximum.
__global__ __launch_bounds__(256) void pref_bound_kernel(PrefParams p) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_pick[4];
  __shared__ float s_max[4];
  const int tid = threadIdx.x;
  const size_t gr = blockIdx.x;
  RowKeys keys;
  keys.load(p.blkmax + gr * p.nblk, (uint32_t)p.nblk);
  uint32_t mk = 0;
  keys.for_each([&](uint32_t key) { mk = max(mk, key); });
  float m = mk != 0 ? key_float(mk) : -INFINITY;
  for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
  if (tid % 64 == 0) s_max[tid / 64] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  float L = -INFINITY;
  if (p.nblk >= p.top_k) L = key_float(kth_largest_key(keys, (uint32_t)p.top_k, hist, s_pick));
  if (tid == 0) {
    p.bound[gr * 2] = L;
    p.bound[gr * 2 + 1] = m;
  }
}

__device__ inline unsigned long long block_sum_u64(unsigned long long v, unsigned long long* scratch) {
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  __syncthreads();
  if (threadIdx.x % 64 == 0) scratch[threadIdx.x / 64] = v;
  __syncthreads();
  return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

// 2^(x scale2 - m) <= 1 as 40-bit fixed point (exact: a float has 24 significant bits); the
// exponent is formed as in pass 2
__device__ inline unsigned long long fixed_mass(float x, float scale2, float minus_m) {
  return (unsigned long long)(__builtin_amdgcn_exp2f(fmaf(x, scale2, minus_m)) * 1099511627776.0f);
}

// One workgroup per row: its share of Eq. 8, 1 - (mass of its top_k largest entries).
__global__ __launch_bounds__(256) void pref_final_kernel(PrefParams p) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_pick[4];
  __shared__ unsigned long long scratch[4];
  const int tid = threadIdx.x;
  const size_t gr = blockIdx.x;
  const uint32_t stored = min(p.cursor[gr * 2], (uint32_t)p.cand_cap);
  const float L = p.bound[gr * 2], minus_m = -p.bound[gr * 2 + 1] * p.scale2;
  const float* cand = p.cand + gr * p.cand_cap;
  const uint32_t k = (uint32_t)p.top_k;
  float result = 0.f;  // a row with at most top_k entries has nothing outside them
  if ((uint32_t)p.n > k) {
    RowKeys keys;
    keys.load(cand, stored);
    float T = L;
    if (stored >= k) T = key_float(kth_largest_key(keys, k, hist, s_pick));
    const uint32_t tkey = float_key(T);
    unsigned long long mass = 0, above = 0;
    keys.for_each([&](uint32_t key) {
      if (key > tkey) mass += fixed_mass(key_float(key), p.scale2, minus_m), above += 1;
    });
    mass = block_sum_u64(mass, scratch);
    above = block_sum_u64(above, scratch);
    mass += (k - above) * fixed_mass(T, p.scale2, minus_m);  // the rest of the top_k entries equal T
    float den = 0.f;
    for (int r = 0; r < p.P; ++r) den += p.den[gr * p.P + r];
    result = den > 0.f ? 1.0f - (float)((double)mass * (1.0 / 1099511627776.0)) / den : 0.f;
  }
  __syncthreads();
  if (tid == 0) {
    p.row_p[gr] = result;
    p.cursor[gr * 2] = 0;
    p.cursor[gr * 2 + 1] = 0;
  }
}

// Eq. 8 per query head: the sum of its rows' shares, in row order (one thread per head).  (A
// launch of its own: an arrival counter per head in the kernel above, 64 atomics on one
// address each, cost three times what this launch does.)
__global__ void pref_sum_kernel(PrefParams p) {
  const int jh = blockIdx.x * blockDim.x + threadIdx.x;  // query head
  if (jh >= p.hq) return;
  float total = 0.f;
  for (int i = 0; i < p.n_q; ++i) total += p.row_p[(size_t)jh * p.n_q + i];  // rows of a KV head: (head of the group, position)
  p.p_out[(size_t)p.b * p.hq + jh] = total;
}

int32_t check_pref_desc(const tkv_pref_desc* d) {
  if (!d || d->struct_size != sizeof(tkv_pref_desc)) return TKV_E_INVAL;
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->batch <= 0 || d->n_q <= 0 || d->top_k <= 0 || d->capacity <= 0)
    return TKV_E_INVAL;
  if (d->n_q_heads % d->n_kv_heads != 0) return TKV_E_INVAL;
  if (d->head_dim != TKV_D || d->batch > TKV_MAX_BATCH) return TKV_E_UNSUPPORTED;
  if (d->n_q % 16 != 0 || d->n_q > 256 || d->top_k > 4096) return TKV_E_UNSUPPORTED;
  return TKV_OK;
}

// How the keys of a prompt of n tokens are shared out (see the kernel's header).
struct PrefSplit {
  int32_t P, rounds, nblk, slabs;
};
int pref_slabs(const tkv_pref_desc* d) { return (d->n_q_heads / d->n_kv_heads * d->n_q + kSlabRows - 1) / kSlabRows; }
// most workgroups per (KV head, slab): the machine filled once
int pref_p_cap(const tkv_pref_desc* d) { return std::max(1, 256 / (d->n_kv_heads * pref_slabs(d))); }
int pref_rounds(int n_chunks, int P) { return ((n_chunks + P - 1) / P + kRound - 1) / kRound; }
PrefSplit pref_split(const tkv_pref_desc* d, int32_t n, int32_t n_cus) {
  PrefSplit sp;
  sp.slabs = pref_slabs(d);
  const int n_chunks = (n + kChunk - 1) / kChunk;
  // fill the machine once, but leave a workgroup a whole round of chunks where the prompt is long
  // enough: blocks of fewer keys make the bound looser (more candidates), never wrong
  int P = std::min(pref_p_cap(d), std::max(1, n_cus / (d->n_kv_heads * sp.slabs)));
  const int by_round = (n_chunks + kRound - 1) / kRound;
  if (P > by_round) P = by_round;
  sp.P = P;
  sp.rounds = pref_rounds(n_chunks, P);
  sp.nblk = P * sp.rounds * kBlocksPerRound;
  return sp;
}

// Workspace of one sequence (sequences are processed one after the other); the counters come
// first: they must be zero before the first call.
struct PrefWs {
  uint32_t* cursor;
  float* blkmax;
  float* bound;
  float* den;
  float* cand;
  float* row_p;
  int32_t cand_cap;
};
size_t pref_ws_layout(const tkv_pref_desc* d, char* base, PrefWs* out) {
  const size_t rows = (size_t)d->n_q_heads * d->n_q;  // Hkv * R
  // the split depends on n and on the stream (its compute units): size for the largest it can be;
  // for a given P the number of blocks grows with n
  const int n_chunks = (d->capacity + kChunk - 1) / kChunk;
  const size_t p_max = (size_t)pref_p_cap(d);
  size_t nblk_max = 0;
  for (int P = 1; P <= (int)p_max; ++P)
    nblk_max = std::max(nblk_max, (size_t)P * pref_rounds(n_chunks, P) * kBlocksPerRound);
  const size_t cand_cap = std::min<size_t>((size_t)d->capacity, (size_t)kBlockKeys * d->top_k);
  size_t o = 0;
  const size_t o_cur = o;    o = tkv::align16(o + rows * 2 * 4);
  const size_t o_blk = o;    o = tkv::align16(o + rows * nblk_max * 4);
  const size_t o_bound = o;  o = tkv::align16(o + rows * 2 * 4);
  const size_t o_den = o;    o = tkv::align16(o + rows * p_max * 4);
  const size_t o_cand = o;   o = tkv::align16(o + rows * cand_cap * 4);
  const size_t o_rowp = o;   o = tkv::align16(o + rows * 4);
  if (out) {
    out->cursor = (uint32_t*)(base + o_cur);
    out->blkmax = (float*)(base + o_blk);
    out->bound = (float*)(base + o_bound);
    out->den = (float*)(base + o_den);
    out->cand = (float*)(base + o_cand);
    out->row_p = (float*)(base + o_rowp);
    out->cand_cap = (int32_t)cand_cap;
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
  if (!(sm_scale > 0.f)) return TKV_E_INVAL;
  if (n > d->capacity) return TKV_E_CAPACITY;
  if (workspace_bytes < pref_ws_layout(d, nullptr, nullptr)) return TKV_E_WORKSPACE;
  PrefWs ws;
  pref_ws_layout(d, (char*)workspace, &ws);
  hipStream_t s = (hipStream_t)stream;
  int n_cus = tkv::stream_compute_units(s);
  if (n_cus > 256) n_cus = 256;
  const PrefSplit sp = pref_split(d, n, n_cus);
  static const bool lds_ok =
      hipFuncSetAttribute(reinterpret_cast<const void*>(&pref_pass_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kPass1Lds) == hipSuccess &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(&pref_pass_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kPass2Lds) == hipSuccess;
  if (!lds_ok) return TKV_E_HIP;
  PrefParams p;
  p.q_last = (const __half*)q_last;
  p.k = (const __half*)k;
  p.blkmax = ws.blkmax;
  p.bound = ws.bound;
  p.den = ws.den;
  p.cand = ws.cand;
  p.cursor = ws.cursor;
  p.row_p = ws.row_p;
  p.p_out = p_out;
  p.scale2 = sm_scale * 1.44269504088896340736f;
  p.hq = d->n_q_heads;
  p.hkv = d->n_kv_heads;
  p.n_q = d->n_q;
  p.n = n;
  p.top_k = d->top_k;
  p.P = sp.P;
  p.rounds = sp.rounds;
  p.nblk = sp.nblk;
  p.cand_cap = ws.cand_cap;
  const int rows = d->n_q_heads * d->n_q;
  const dim3 grid(sp.P, d->n_kv_heads, sp.slabs);
  for (int b = 0; b < d->batch; ++b) {
    p.b = b;
    TKV_LAUNCH(pref_pass_kernel<1>, grid, kThreads, kPass1Lds, s, p);
    TKV_LAUNCH(pref_bound_kernel, dim3(rows), 256, 0, s, p);
    TKV_LAUNCH(pref_pass_kernel<2>, grid, kThreads, kPass2Lds, s, p);
    TKV_LAUNCH(pref_final_kernel, dim3(rows), 256, 0, s, p);
    TKV_LAUNCH(pref_sum_kernel, dim3((d->n_q_heads + 63) / 64), 64, 0, s, p);
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
