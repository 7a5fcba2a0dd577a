// Internal helpers shared by the tkv HIP sources (gfx950 only).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "tkv.h"
#include "tkv_debug.h"

#define TKV_D 128      // head_dim
#define TKV_BLK 32     // tokens per block of packed codes (the quantization group is 32 or 64)
#define TKV_WAVE 64

// Partial attention result of one chunk and one query head, in floats: max logit (in log2
// units after scaling), sum of weights, two unused words, then the weighted V sum (so that
// it starts on a 16-byte boundary).
#define TKV_PART_O 4
#define TKV_PART_STRIDE (TKV_D + TKV_PART_O)

// Upper bound on split-K chunks per (sequence, KV head), tail chunk excluded.
#define TKV_MAX_CHUNKS 256

#define TKV_HIP_TRY(expr)                      \
  do {                                         \
    hipError_t _e = (expr);                    \
    if (_e != hipSuccess) return TKV_E_HIP;    \
  } while (0)

struct TkvSeqLens {
  int32_t n[TKV_MAX_BATCH];
};

namespace tkv {

// The new tokens of a step that a quantized layer's attention call also appends:
// k_new, v_new fp16 [B][n_stride][Hkv][D], the first n_add[b] rows of sequence b.
struct QuantNewTokens {
  const __half* k_new;
  const __half* v_new;
  int32_t n_stride;
  TkvSeqLens n_add;
};

// Number of quantized tokens of a sequence of n tokens (residual w, group g).
__host__ __device__ inline int32_t n_quantized(int32_t n, int32_t w, int32_t g) {
  return n >= w ? ((n - w) / g) * g : 0;
}

// Kernel launch whose status is the launch's own return value: the process-wide "last error" of
// the HIP runtime is neither read nor cleared, so an earlier error of the calling program is
// never reported as the library's and never erased.
template <typename... KArgs, typename... Args>
inline int32_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t s,
                      Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "kernel argument count");
  std::tuple<KArgs...> vals{static_cast<KArgs>(std::forward<Args>(args))...};
  void* ptrs[sizeof...(KArgs)];
  std::apply([&](auto&... v) { int i = 0; ((ptrs[i++] = (void*)&v), ...); }, vals);
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, s) == hipSuccess
             ? TKV_OK
             : TKV_E_HIP;
}
#define TKV_LAUNCH(kernel, grid, block, lds, stream, ...)                                                  \
  do {                                                                                                     \
    if (tkv::launch(kernel, grid, block, lds, stream, __VA_ARGS__) != TKV_OK) return TKV_E_HIP;            \
  } while (0)

// Compute units that kernels of this stream may use: those of its compute-unit mask
// (hipExtStreamCreateWithCUMask), all of the device's for an ordinary stream.  Launches that
// aim at one workgroup per compute unit size themselves with it.
inline int stream_compute_units(hipStream_t s) {
  static const int device_cus = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      v = 0;
    return v > 0 ? v : 256;
  }();
  uint32_t mask[16] = {0};
  if (hipExtStreamGetCUMask(s, 16, mask) != hipSuccess) {
    (void)hipGetLastError();
    return device_cus;
  }
  int cus = 0;
  for (uint32_t m : mask) cus += __builtin_popcount(m);
  return cus > 0 && cus <= device_cus ? cus : device_cus;
}

int32_t check_quant_desc(const tkv_quant_desc* d);
// Merges [n_heads_total][n_parts][TKV_PART_STRIDE] float partials (max in log2 units, sum,
// weighted V) into fp16 [n_heads_total][D].
int32_t launch_attn_merge(const float* parts, __half* out, int n_heads_total, int n_parts, hipStream_t s);
int32_t check_sparse_desc(const tkv_sparse_desc* d);

// Device-visible address of a caller's buffer.  kDevHostOnly: pinned host memory only
// (TKV_E_NOTPINNED otherwise); kDevAny: pinned host memory or device memory; kDevDeviceOnly:
// device memory only (TKV_E_INVAL otherwise).
enum DevView { kDevHostOnly, kDevAny, kDevDeviceOnly };
inline int32_t device_view(const void* ptr, DevView mode, const void** dev) {
  hipPointerAttribute_t attr;
  const hipError_t e = hipPointerGetAttributes(&attr, ptr);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    if (mode == kDevDeviceOnly) return TKV_E_INVAL;
    return e == hipErrorInvalidValue ? TKV_E_NOTPINNED : TKV_E_HIP;
  }
  if (attr.type == hipMemoryTypeDevice) {
    if (mode == kDevHostOnly) return TKV_E_NOTPINNED;
    *dev = ptr;
    return TKV_OK;
  }
  if (mode == kDevDeviceOnly) return TKV_E_INVAL;
  if (attr.type != hipMemoryTypeHost || attr.devicePointer == nullptr) return TKV_E_NOTPINNED;
  *dev = attr.devicePointer;
  return TKV_OK;
}

// ---- cross-chunk merge by the last workgroup of a (sequence, KV head) --------------------
// Partials cross workgroups through device-scope stores and loads (they bypass the caches
// that are not coherent between workgroups).  Such loads are served slowly, one load
// instruction after the other, so the merge uses as few and as wide ones as it can: all of
// them are issued before the first is used.  The partial maximum and sum of a chunk sit next
// to each other (one 8-byte load), the weighted V sum starts on a 16-byte boundary.

typedef float tkv_floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t tkv_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t tkv_u32x2 __attribute__((ext_vector_type(2)));

// Device-scope loads of 4, 8 or 16 bytes through a buffer descriptor over [base, base + bytes)
// (base must be uniform over the wave; byte offsets are 32 bit).  The "sc1" cache policy makes
// them device-scope like an agent-scope atomic load, but up to 16 bytes wide, and the compiler
// itself tracks when their results arrive.  An offset at or beyond `bytes` reads nothing and
// returns 0, which spares the callers a branch around loads they do not need (kNone).
struct AgentBuf {
  static constexpr uint32_t kNone = 0xFFFFFFF0u;
  __amdgpu_buffer_rsrc_t r;
  __device__ AgentBuf(const void* base, uint32_t bytes)
      : r(__builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000)) {}
  __device__ tkv_u32x4 x4(uint32_t off) const { return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 16); }
  __device__ tkv_u32x2 x2(uint32_t off) const { return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 16); }
  __device__ uint32_t x1(uint32_t off) const { return __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 16); }
};

// head0: partials of the G heads of this KV head, [G][n_chunks][TKV_PART_STRIDE]; out0: fp16
// [G][128].  lds: 3 * G * n_chunks + 4 * 4 * 128 + 4 floats.  Called by every thread of the
// workgroup (nthr a multiple of 64, at least 64 * G).
__device__ inline void merge_chunks(const float* head0, int G, int n_chunks, __half* out0, float* lds, int tid,
                                    int nthr) {
  float* ml = lds;                       // [G][n_chunks][2]
  float* cw = ml + 2 * G * n_chunks;     // [G][n_chunks] weights
  float* red = cw + G * n_chunks;        // [4 heads][4 classes][128]
  float* Ls = red + 4 * 4 * TKV_D;       // [4]
  const int lane = tid % 64, wave = tid / 64;
  const AgentBuf pb(head0, (uint32_t)((size_t)G * n_chunks * TKV_PART_STRIDE * sizeof(float)));
  // first pass: maxima and sums of all chunks, and (for up to 64 chunks) this thread's channels
  for (int i = tid; i < G * n_chunks; i += nthr) {
    const tkv_u32x2 v = pb.x2((uint32_t)i * TKV_PART_STRIDE * 4u);
    // (elements copied out before the cast: a bit cast applied directly to a vector element
    // reads element 0 with this compiler)
    const uint32_t v_max = v.x, v_sum = v.y;
    ml[2 * i] = __uint_as_float(v_max);
    ml[2 * i + 1] = __uint_as_float(v_sum);
  }
  // item = (head, chunk class ks, channel quad c4): chunks ks, ks + 4, ...
  constexpr int kPer = 16;
  for (int item0 = 0; item0 < G * TKV_D; item0 += nthr) {
    const int item = item0 + tid;
    const bool on = item < G * TKV_D;
    const int hh = on ? item / TKV_D : 0, r = item % TKV_D;
    const int ks = r / 32, c4 = r % 32;
    const uint32_t base = (uint32_t)((hh * n_chunks) * TKV_PART_STRIDE + TKV_PART_O + 4 * c4) * 4u;
    tkv_floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < n_chunks; k0 += 4 * kPer) {
      tkv_u32x4 ov[kPer];
#pragma unroll
      for (int y = 0; y < kPer; ++y) {
        const int k = k0 + 4 * y + ks;
        ov[y] = pb.x4(on && k < n_chunks ? base + (uint32_t)k * TKV_PART_STRIDE * 4u : AgentBuf::kNone);
      }
      if (item0 == 0 && k0 == 0) {
        // weights: one wave per head (the loads above are in flight meanwhile)
        __syncthreads();
        if (wave < G) {
          float M = -INFINITY;
          for (int k = lane; k < n_chunks; k += 64) M = fmaxf(M, ml[2 * (wave * n_chunks + k)]);
          for (int m = 32; m >= 1; m >>= 1) M = fmaxf(M, __shfl_xor(M, m, 64));
          float Lsum = 0.f;
          for (int k = lane; k < n_chunks; k += 64) {
            const float mk = ml[2 * (wave * n_chunks + k)];
            const float w = mk == -INFINITY ? 0.f : exp2f(mk - M);
            cw[wave * n_chunks + k] = w;
            Lsum = __builtin_fmaf(ml[2 * (wave * n_chunks + k) + 1], w, Lsum);
          }
          for (int m = 32; m >= 1; m >>= 1) Lsum += __shfl_xor(Lsum, m, 64);
          if (lane == 0) Ls[wave] = Lsum;
        }
        __syncthreads();
      }
#pragma unroll
      for (int y = 0; y < kPer; ++y) {
        const int k = k0 + 4 * y + ks;
        const float w = (on && k < n_chunks) ? cw[hh * n_chunks + k] : 0.f;
        acc += __builtin_bit_cast(tkv_floatx4, ov[y]) * w;
      }
    }
    if (on) *reinterpret_cast<tkv_floatx4*>(red + (hh * 4 + ks) * TKV_D + 4 * c4) = acc;
  }
  __syncthreads();
  for (int i = tid; i < G * TKV_D; i += nthr) {
    const int hh = i / TKV_D, c = i % TKV_D;
    const float O = (red[(hh * 4 + 0) * TKV_D + c] + red[(hh * 4 + 1) * TKV_D + c]) +
                    (red[(hh * 4 + 2) * TKV_D + c] + red[(hh * 4 + 3) * TKV_D + c]);
    const float Lsum = Ls[hh];
    out0[(size_t)hh * TKV_D + c] = __float2half_rn(Lsum > 0.f ? O / Lsum : 0.f);
  }
}

// Eq. 10 (Sec. 4.2, Stage 1) for one (sequence, KV head), by a whole workgroup of at least
// TKV_D threads (thread c < TKV_D owns channel c; contains barriers):
//   s_c = (((|q_0,c| + |q_1,c|) + ...) over the G query heads) * kmax[c],
// every operation one float32 operation; the ds channels with the largest s (ties: lower
// channel first) go to out[0..ds) in ascending order (and to out2 unless null).
// q0: the G query rows [G][TKV_D]; s_s, s_sel: TKV_D words of LDS scratch each.
__device__ inline void select_channels_block(const __half* q0, int G, const float* kmax, int ds, float* s_s,
                                             uint32_t* s_sel, int32_t* out, int32_t* out2) {
#pragma clang fp contract(off)
  const int c = threadIdx.x;
  float s = 0.f;
  if (c < TKV_D) {
    float a = fabsf(__half2float(q0[c]));
    for (int j = 1; j < G; ++j) a = a + fabsf(__half2float(q0[(size_t)j * TKV_D + c]));
    s = a * kmax[c];
    s_s[c] = s;
  }
  __syncthreads();
  bool sel = false;
  if (c < TKV_D) {
    int rank = 0;  // channels that come before this one: larger s, or equal s and lower index
    for (int j = 0; j < TKV_D; ++j) {
      const float sj = s_s[j];
      rank += (sj > s || (sj == s && j < c)) ? 1 : 0;
    }
    sel = rank < ds;
    s_sel[c] = sel ? 1u : 0u;
  }
  __syncthreads();
  if (sel) {
    int pos = 0;  // ascending output: selected channels below this one
    for (int j = 0; j < c; ++j) pos += (int)s_sel[j];
    out[pos] = c;
    if (out2) out2[pos] = c;
  }
  __syncthreads();
}

// Carve-up of the sparse-layer workspace (per bh = (sequence, KV head)):
//   keys  uint32 [BH][capacity]   order-preserving image of the approximate scores
//   cand  uint2  [BH][capacity + 4096]  (key, token) pairs in or above the threshold bin; the
//                                 workgroup that owns tokens [T x, T x + T) lists them from entry T x
//                                 (T = tokens per workgroup of the launch, rounded up to 4)
//   hist  uint32 [BH][8192]       histogram of the 13-bit key prefix
//   ctrl  uint32 [BH][8]          1: arrival counter of the Top-K selection; 4: arrival counter of
//                                 the attention
//   blk   uint32 [BH][nblk_cap]   length of each workgroup's list
//   parts float  [B][Hq][64][D+4] split partials of the sparse attention
struct SparseWs {
  uint32_t* keys;
  uint2* cand;
  size_t cand_stride;  // entries per (sequence, KV head)
  uint32_t* hist;
  uint32_t* ctrl;
  uint32_t* blk;
  float* parts;
  int32_t nblk_cap;
};
inline size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }
inline size_t sparse_ws_layout(const tkv_sparse_desc* d, size_t off[6], int32_t* nblk_cap) {
  const size_t bh = (size_t)d->batch * d->n_kv_heads, cap = (size_t)d->capacity;
  const int32_t nb = (int32_t)((cap + 1023) / 1024 + 1);
  size_t o = 0;
  off[0] = o; o = align16(o + bh * cap * 4);
  off[1] = o; o = align16(o + bh * (cap + 4096) * 8);
  off[2] = o; o += bh * 8192 * 4;
  off[3] = o; o = align16(o + bh * 8 * 4);
  off[4] = o; o = align16(o + bh * (size_t)nb * 4);
  off[5] = o; o = align16(o + (size_t)d->batch * d->n_q_heads * 64 * TKV_PART_STRIDE * 4);
  if (nblk_cap) *nblk_cap = nb;
  return o;
}
inline SparseWs carve_sparse_ws(const tkv_sparse_desc* d, void* workspace) {
  size_t off[6];
  SparseWs ws;
  sparse_ws_layout(d, off, &ws.nblk_cap);
  char* base = (char*)workspace;
  ws.keys = (uint32_t*)(base + off[0]);
  ws.cand = (uint2*)(base + off[1]);
  ws.cand_stride = (size_t)d->capacity + 4096;
  ws.hist = (uint32_t*)(base + off[2]);
  ws.ctrl = (uint32_t*)(base + off[3]);
  ws.blk = (uint32_t*)(base + off[4]);
  ws.parts = (float*)(base + off[5]);
  return ws;
}

// Position of logical element (t, c) of a block of 32 tokens x 128 channels inside the
// packed block: word index and field index.  Mirrors the layout text of tkv.h.
__host__ __device__ inline void k_code_pos(int bits, int t, int c, int& word, int& field) {
  const int r = 4 * (t / 8) + t % 4, tau = (t % 8) / 4;
  const int lane = r + 16 * ((c % 32) / 8);
  if (bits == 1) {
    word = 64 * tau + lane;
    field = (c % 8) / 2 + 4 * ((c / 32) % 2) + 8 * (c / 64) + 16 * (c % 2);
  } else if (bits == 2) {
    word = 4 * lane + 2 * tau + c / 64;
    field = (c % 8) / 2 + 4 * ((c / 32) % 2) + 8 * (c % 2);
  } else {
    word = 256 * tau + 4 * lane + c / 32;
    field = (c % 8) / 2 + 4 * (c % 2);
  }
}

__host__ __device__ inline void v_code_pos(int bits, int t, int c, int& word, int& field) {
  const int lane = c % 16 + 16 * (t / 8);
  if (bits == 1) {
    word = 64 * (c / 64) + lane;
    field = (t % 8) / 2 + 4 * ((c / 16) % 2) + 8 * ((c / 32) % 2) + 16 * (t % 2);
  } else if (bits == 2) {
    word = 4 * lane + c / 32;
    field = (t % 8) / 2 + 4 * ((c / 16) % 2) + 8 * (t % 2);
  } else {
    word = 256 * (c / 64) + 4 * lane + (c / 16) % 4;
    field = (t % 8) / 2 + 4 * (t % 2);
  }
}

// Inverse maps: which (t, c) does field F of word w hold.
__host__ __device__ inline void k_code_elem(int bits, int w, int F, int& t, int& c) {
  int lane, tau, r, kb;
  if (bits == 1) {
    tau = w / 64;
    lane = w % 64;
    const int f = F % 16, e = F / 16;
    r = lane % 16;
    kb = lane / 16;
    c = 32 * ((f / 4) % 2) + 64 * (f / 8) + 8 * kb + 2 * (f % 4) + e;
  } else if (bits == 2) {
    lane = w / 4;
    tau = (w % 4) / 2;
    const int wd = w % 2, f = F % 8, e = F / 8;
    r = lane % 16;
    kb = lane / 16;
    c = 64 * wd + 32 * (f / 4) + 8 * kb + 2 * (f % 4) + e;
  } else {
    tau = w / 256;
    lane = (w % 256) / 4;
    const int m = w % 4, f = F % 4, e = F / 4;
    r = lane % 16;
    kb = lane / 16;
    c = 32 * m + 8 * kb + 2 * f + e;
  }
  t = 8 * (r / 4) + 4 * tau + r % 4;
}

__host__ __device__ inline void v_code_elem(int bits, int w, int F, int& t, int& c) {
  if (bits == 1) {
    const int lane = w % 64, f = F % 16, e = F / 16;
    const int r = lane % 16, kb = lane / 16;
    const int cb = 4 * (w / 64) + (f / 4) % 2 + 2 * (f / 8);
    t = 8 * kb + 2 * (f % 4) + e;
    c = 16 * cb + r;
  } else if (bits == 2) {
    const int lane = w / 4, wd = w % 4, f = F % 8, e = F / 8;
    const int r = lane % 16, kb = lane / 16;
    const int cb = 2 * wd + f / 4;
    t = 8 * kb + 2 * (f % 4) + e;
    c = 16 * cb + r;
  } else {
    const int lam = w / 256, lane = (w % 256) / 4, f = F % 4, e = F / 4;
    const int r = lane % 16, kb = lane / 16;
    const int cb = 4 * lam + w % 4;
    t = 8 * kb + 2 * f + e;
    c = 16 * cb + r;
  }
}

}  // namespace tkv
