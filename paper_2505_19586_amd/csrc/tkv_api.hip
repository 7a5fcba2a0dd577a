// Status strings, descriptor validation and buffer-size helpers of the tkv C ABI.
#include "tkv_common.h"

extern "C" const char* tkv_strerror(int32_t status) {
  switch (status) {
    case TKV_OK: return "ok";
    case TKV_E_INVAL: return "invalid argument";
    case TKV_E_UNSUPPORTED: return "configuration not supported by the gfx950 kernels";
    case TKV_E_CAPACITY: return "sequence length exceeds cache capacity";
    case TKV_E_WORKSPACE: return "workspace too small";
    case TKV_E_NOTPINNED: return "kv_host is not device-accessible pinned host memory";
    case TKV_E_HIP: return "HIP runtime error";
    default: return "unknown tkv status";
  }
}

namespace tkv {

// Up to 8 query heads per KV head.
static int32_t check_heads(int32_t hq, int32_t hkv, int32_t d, int32_t batch) {
  if (hq <= 0 || hkv <= 0 || d <= 0 || batch <= 0) return TKV_E_INVAL;
  if (hq % hkv != 0) return TKV_E_INVAL;
  if (batch > TKV_MAX_BATCH) return TKV_E_UNSUPPORTED;
  if (d != TKV_D) return TKV_E_UNSUPPORTED;
  if (hq / hkv > 8) return TKV_E_UNSUPPORTED;
  return TKV_OK;
}

int32_t check_quant_desc(const tkv_quant_desc* d) {
  if (!d || d->struct_size != sizeof(tkv_quant_desc)) return TKV_E_INVAL;
  int32_t st = check_heads(d->n_q_heads, d->n_kv_heads, d->head_dim, d->batch);
  if (st != TKV_OK) return st;
  if (d->group_size <= 0 || d->residual < 0 || d->capacity <= 0 || d->bits <= 0) return TKV_E_INVAL;
  if (d->bits != 1 && d->bits != 2 && d->bits != 4) return TKV_E_UNSUPPORTED;
  if (d->group_size != 32 && d->group_size != 64) return TKV_E_UNSUPPORTED;
  if (d->residual % d->group_size != 0 || d->capacity % d->group_size != 0) return TKV_E_INVAL;
  if (d->residual < d->group_size || d->residual + d->group_size > 1024) return TKV_E_UNSUPPORTED;
  return TKV_OK;
}

int32_t check_sparse_desc(const tkv_sparse_desc* d) {
  if (!d || d->struct_size != sizeof(tkv_sparse_desc)) return TKV_E_INVAL;
  int32_t st = check_heads(d->n_q_heads, d->n_kv_heads, d->head_dim, d->batch);
  if (st != TKV_OK) return st;
  if (d->n_channels <= 0 || d->top_k <= 0 || d->n_sink < 0 || d->n_window <= 0 || d->capacity <= 0)
    return TKV_E_INVAL;
  if (d->n_channels != 16 && d->n_channels != 12 && d->n_channels != 8) return TKV_E_UNSUPPORTED;
  if (d->top_k > 4096 || d->n_window > 1024 || d->n_sink > 1024) return TKV_E_UNSUPPORTED;
  return TKV_OK;
}

}  // namespace tkv

extern "C" int32_t tkv_quant_cache_sizes(const tkv_quant_desc* d, size_t bytes_out[8], size_t* workspace_bytes) {
  int32_t st = tkv::check_quant_desc(d);
  if (st != TKV_OK) return st;
  const size_t bh = (size_t)d->batch * d->n_kv_heads;
  const size_t cap = (size_t)d->capacity;
  const size_t codes = bh * cap * TKV_D * d->bits / 8;
  const size_t g = (size_t)d->group_size;
  const size_t kmeta = bh * (cap / g) * TKV_D * 2;
  const size_t vmeta = bh * cap * (TKV_D / g) * 2;
  const size_t resid = bh * ((size_t)d->residual + g) * TKV_D * 2;
  if (bytes_out) {
    bytes_out[0] = codes;
    bytes_out[1] = kmeta;
    bytes_out[2] = kmeta;
    bytes_out[3] = codes;
    bytes_out[4] = vmeta;
    bytes_out[5] = vmeta;
    bytes_out[6] = resid;
    bytes_out[7] = resid;
  }
  if (workspace_bytes) {
    // split-K partials: [B][Hq][chunks + tail][D + 4] float, plus one arrival
    // counter per (sequence, KV head, four query heads of its group)
    *workspace_bytes = (size_t)d->batch * d->n_q_heads * (TKV_MAX_CHUNKS + 1) * TKV_PART_STRIDE * sizeof(float) +
                       2 * bh * sizeof(uint32_t) + 512;
  }
  return TKV_OK;
}

extern "C" int32_t tkv_sparse_cache_sizes(const tkv_sparse_desc* d, size_t bytes_out[4], size_t* workspace_bytes) {
  int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  const size_t bh = (size_t)d->batch * d->n_kv_heads;
  const size_t cap = (size_t)d->capacity;
  if (bytes_out) {
    bytes_out[0] = bh * cap * d->n_channels * 2;
    bytes_out[1] = bh * d->n_channels * sizeof(int32_t);
    bytes_out[2] = bh * cap * 2 * TKV_D * 2;
    bytes_out[3] = bh * (size_t)(d->n_sink + d->n_window) * 2 * TKV_D * 2;
  }
  if (workspace_bytes) {
    // Top-K scratch and attention partials; layout in tkv_common.h
    size_t off[6];
    *workspace_bytes = tkv::sparse_ws_layout(d, off, nullptr) + 256;
  }
  return TKV_OK;
}

namespace {

// Measurement aid: a plain read sweep of a device buffer, 16 bytes per lane and load, eight
// loads in flight per lane.  The loaded words are folded into one value that is stored only
// if it equals a constant no fold produces in practice, so the loads cannot be dropped.
__global__ __launch_bounds__(256) void read_sweep_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint32_t acc = 0u;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = src[i + j * stride];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  for (; i < n16; i += stride) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u && sink) sink[blockIdx.x] = acc;
}

}  // namespace

extern "C" int32_t tkv_debug_read_sweep(const void* src, size_t bytes, void* sink, int32_t n_workgroups, void* stream) {
  if (!src || bytes == 0 || bytes % 16 != 0 || ((uintptr_t)src & 15) != 0) return TKV_E_INVAL;
  if (n_workgroups <= 0 || n_workgroups > 65536) return TKV_E_INVAL;
  TKV_LAUNCH(read_sweep_kernel, dim3(n_workgroups), 256, 0, (hipStream_t)stream, (const uint4*)src, bytes / 16, (uint32_t*)sink);
  return TKV_OK;
}

extern "C" int32_t tkv_debug_quant_workspace(const tkv_quant_desc* d, size_t* scratch_bytes) {
  const int32_t st = tkv::check_quant_desc(d);
  if (st != TKV_OK) return st;
  if (!scratch_bytes) return TKV_E_INVAL;
  *scratch_bytes = (size_t)d->batch * d->n_q_heads * (TKV_MAX_CHUNKS + 1) * TKV_PART_STRIDE * sizeof(float);
  return TKV_OK;
}

extern "C" int32_t tkv_debug_sparse_workspace(const tkv_sparse_desc* d, size_t region_offsets[7]) {
  const int32_t st = tkv::check_sparse_desc(d);
  if (st != TKV_OK) return st;
  if (!region_offsets) return TKV_E_INVAL;
  size_t off[6];
  region_offsets[6] = tkv::sparse_ws_layout(d, off, nullptr);
  for (int i = 0; i < 6; ++i) region_offsets[i] = off[i];
  return TKV_OK;
}
