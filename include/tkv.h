/*
 * tkv - decode-time attention of TailorKV's hybrid KV cache (arxiv 2505.19586)
 * for AMD MI355X (gfx950).  C ABI.
 *
 * Two kinds of layers (Sec. 4.1 of the paper):
 *   - quantization-friendly layers keep the whole cache on the GPU, quantized with
 *     the uniform asymmetric quantizer of Sec. 2.2 (Eq. 4), keys per channel and
 *     values per token (Sec. 4.3), zero-point and scaler in fp16 (Sec. 4.4);
 *   - sparsity-friendly layers keep the full fp16 cache in pinned host memory and a
 *     small critical-key summary on the GPU; each decode step scores every cached
 *     token approximately, takes the Top-K, fetches only those tokens' K/V rows from
 *     the host and attends exactly over n_local + n_topk tokens (Sec. 4.2, Sec. 5.1).
 *
 * Conventions
 *   - Every function returns a tkv_status (0 = ok, negative = error).  Argument
 *     errors are reported before anything is enqueued and never touch the GPU.
 *   - The caller owns every buffer.  Unless an argument says "host", pointers are
 *     device pointers.  The library allocates no memory.  What it keeps between calls:
 *     a few cached device queries (process-wide), and per HOST THREAD two events that
 *     tkv_sparse_gather_attn uses to order its two streams (created at that thread's
 *     first two-stream call, never destroyed).  Calls from different host threads are
 *     independent as long as they use different workspaces and streams.
 *   - A returned TKV_E_HIP comes from a HIP call the library made itself; the
 *     library neither reads nor clears the runtime's process-wide "last error".
 *   - Calls enqueue work on the given hipStream_t (passed as void*) and return
 *     without synchronizing.  Sequence lengths live in caller-owned HOST int32
 *     arrays; kernels receive them by value, so the arrays may be changed as soon as
 *     a call returns.  At most TKV_MAX_BATCH sequences per call.
 *   - fp16 is IEEE binary16 everywhere.  head_dim must be 128, the quantization
 *     group g 32 or 64.  n_q_heads / n_kv_heads: any number from 1 to 8 (quantized layers:
 *     the attention kernels take a group 4 query heads at a time, and the parts of a group
 *     of 5 to 8 read the codes once each; sparse layers: a row is fetched once whatever the
 *     group; tkv_sparse_decode is one launch for groups of up to 4 and two above); any number
 *     for the dense preference score.
 *   - Token t of sequence b, KV head h.  "group j" is tokens [g j, g j + g); codes are
 *     stored in "blocks" of 32 tokens whatever g is.
 */
#ifndef TKV_H
#define TKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TKV_MAX_BATCH 64

typedef enum {
  TKV_OK = 0,
  TKV_E_INVAL = -1,       /* NULL pointer, bad struct_size, inconsistent shapes            */
  TKV_E_UNSUPPORTED = -2, /* valid request the kernels are not built for (bits, dims, ...) */
  TKV_E_CAPACITY = -3,    /* sequence length would exceed the cache capacity               */
  TKV_E_WORKSPACE = -4,   /* workspace smaller than tkv_*_cache_sizes reports              */
  TKV_E_NOTPINNED = -5,   /* kv_host is not device-accessible pinned host memory           */
  TKV_E_HIP = -6          /* a HIP runtime call failed (also: no usable GPU)               */
} tkv_status;

const char* tkv_strerror(int32_t status);

/* ---------------------------------------------------------------------------------
 * Quantization-friendly layers
 * ------------------------------------------------------------------------------- */

typedef struct {
  uint32_t struct_size; /* sizeof(tkv_quant_desc)                                        */
  int32_t n_q_heads;    /* Hq                                                            */
  int32_t n_kv_heads;   /* Hkv; query head i reads KV head i / (Hq/Hkv)                  */
  int32_t head_dim;     /* D = 128                                                       */
  int32_t bits;         /* b = 1, 2 or 4 (Eq. 4); Sec. 5.1 runs 1 and 2                  */
  int32_t group_size;   /* g = 32 or 64 (Sec. 5.1: 64): tokens per key group, channels
                           per value group                                               */
  int32_t residual;     /* W: newest tokens kept fp16; multiple of g, g <= W <= 1024 - g */
  int32_t capacity;     /* max tokens per sequence, multiple of g                        */
  int32_t batch;        /* B, 1..TKV_MAX_BATCH                                           */
} tkv_quant_desc;

/*
 * Cache buffers of one layer.  With N tokens in a sequence, the first
 * Nq = g*floor((N-W)/g) (0 if N < W) are quantized, the last N-Nq (W..W+g-1 once
 * N >= W) are fp16 in a ring: token t >= Nq sits at ring slot t mod (W+g).
 *
 * Packed layouts (J = capacity/32 blocks of 32 tokens; t = token inside its block,
 * c = channel; a code takes `bits` bits at field F, i.e. bits [bits*F, bits*F+bits)
 * of a little-endian 32-bit word).  The order inside a block is the order in which a
 * wave64 feeds 16x16x32 matrix-core operands from its loads.
 *
 *  k_codes uint32 [B][Hkv][J][32*128*bits/32 words]
 *    1 bit: word = 64*tau + lane, F = (c%8)/2 + 4*((c/32)%2) + 8*(c/64) + 16*(c%2)
 *           (r, tau, lane as for 2 bit)
 *    2 bit: word = 4*lane + 2*tau + wd,  F = f + 8*e, with
 *           r = 4*(t/8) + t%4, tau = (t%8)/4, lane = r + 16*((c%32)/8),
 *           wd = c/64, f = (c%8)/2 + 4*((c/32)%2), e = c%2
 *    4 bit: word = 256*tau + 4*lane + c/32, F = (c%8)/2 + 4*(c%2)   (r, tau, lane as above)
 *  v_codes uint32 [B][Hkv][J][32*128*bits/32 words]
 *    1 bit: word = 64*(c/64) + lane, F = (t%8)/2 + 4*((c/16)%2) + 8*((c/32)%2) + 16*(t%2)
 *           (lane as for 2 bit)
 *    2 bit: word = 4*lane + wd, F = f + 8*e, with
 *           lane = c%16 + 16*(t/8), wd = c/32, f = (t%8)/2 + 4*((c/16)%2), e = t%2
 *    4 bit: word = 256*(c/64) + 4*lane + (c/16)%4, F = (t%8)/2 + 4*(t%2)
 *  k_scale, k_zero  fp16 [B][Hkv][capacity/g][128]   one (s, z) per group and channel
 *  v_scale, v_zero  fp16 [B][Hkv][J][128/g][32]       one (s, z) per token and g-channel
 *                                                     group u = c/g, stored per block [u][t]
 *  k_resid, v_resid fp16 [B][Hkv][W+g][128]    ring of unquantized tokens
 */
typedef struct {
  void* k_codes;
  void* k_scale;
  void* k_zero;
  void* v_codes;
  void* v_scale;
  void* v_zero;
  void* k_resid;
  void* v_resid;
  int32_t* seq_len_host; /* HOST int32 [B]: tokens in each sequence; append updates it */
} tkv_quant_cache;

/*
 * Bytes of each tkv_quant_cache buffer in field order (k_codes ... v_resid) and of
 * the workspace tkv_quant_attn_decode needs.  The code and scaler/zero-point bytes
 * add up to the memory model of Sec. 4.4, Table 2: 2*n*h*d_h*(b/16 + 2/g) fp16
 * elements per layer.  Either output pointer may be NULL.
 */
int32_t tkv_quant_cache_sizes(const tkv_quant_desc* desc, size_t bytes_out[8], size_t* workspace_bytes);

/*
 * Sec. 2.1 Eq. 2 (cache update) + Sec. 2.2 Eq. 4 / Sec. 4.3 (static quantization).
 * Appends n_new tokens to every sequence: k_new, v_new fp16 [B][n_new][Hkv][128]
 * (device).  Every token group that becomes complete and older than the residual is
 * quantized: keys per channel over the group's g tokens, values per token over each
 * g-channel group, with
 *     z = min X (stored as is), s = fp16( (f32(max X) - f32(min X)) / f32(2^b - 1) ),
 *     code = clamp( rint( (f32(x) - f32(z)) / f32(s) ), 0, 2^b - 1 ), rint ties-to-even,
 *     code = 0 where the stored s is 0,
 * every operation a single float32 operation.  seq_len_host[b] += n_new on success.
 * n_new == 0 is a no-op.  Errors: TKV_E_CAPACITY if any seq_len + n_new > capacity.
 */
int32_t tkv_quantize_append(const tkv_quant_desc* desc, tkv_quant_cache* cache, const void* k_new,
                            const void* v_new, int32_t n_new, void* stream);

/* Same, for a padded batch: k_new, v_new hold n_new rows per sequence of which only
 * the first n_valid_host[b] (HOST int32 [B], 0 <= n_valid <= n_new) are appended to
 * sequence b.  n_valid_host == NULL means n_new for every sequence. */
int32_t tkv_quantize_append_ragged(const tkv_quant_desc* desc, tkv_quant_cache* cache, const void* k_new,
                                   const void* v_new, int32_t n_new, const int32_t* n_valid_host, void* stream);

/*
 * Sec. 2.1 Eq. 3 over the dequantized cache (Sec. 4.3): for every query head,
 * logits = sm_scale * q . (code*s + z) over the quantized tokens and sm_scale * q . k
 * over the fp16 tail, one softmax over all N tokens, out = weights . V-hat.
 * q, out: fp16 [B][Hq][128].  A sequence with 0 tokens yields zeros.
 * Input range: the matrix-core kernel feeds fp16 products to the matrix cores: softmax
 * weight x value scaler, and query element x key scaler.  Cached values of magnitude up
 * to about 1000 and query-times-key-scaler products up to 65504 are safe at every bit
 * width; far larger ones overflow fp16 and give wrong or non-finite outputs (the
 * reference kernel that tkv_debug.h can switch to has no such limit).
 * Context length: the rounding error of the matrix-core path grows slowly with the number of
 * tokens (the softmax weights enter the matrix cores as fp16); against a float64 evaluation it
 * measures 5e-4 .. 1e-3 up to 32768 tokens, 1.0e-3 .. 1.5e-3 at 131072 and at 262144, the
 * largest length the parity tests cover (bound 2e-3).
 * Two calls on the same inputs can differ in the last bits of an output (up to about 8e-4 of a
 * head's largest output): which 32-token blocks a wave processes is decided at run time.
 * The work is split over token chunks whose partial (max, sum, weighted V) results
 * go through `workspace` and are merged with a log-sum-exp merge.  The workspace must be
 * ZERO-FILLED by the caller before its first use (it ends in arrival counters that every
 * call leaves zero); concurrent calls need separate workspaces.
 */
int32_t tkv_quant_attn_decode(const tkv_quant_desc* desc, const tkv_quant_cache* cache, const void* q,
                              void* out, float sm_scale, void* workspace, size_t workspace_bytes,
                              void* stream);

/*
 * The decode step of a quantization-friendly layer in one call: Eq. 2 (the step's new tokens
 * join the cache, as tkv_quantize_append_ragged with the same k_new, v_new, n_new,
 * n_valid_host) and then Eq. 3 over the grown cache (as tkv_quant_attn_decode with the same q,
 * out, sm_scale, workspace).  Same cache contents, same seq_len_host and the same results (to
 * tkv_quant_attn_decode's run-to-run variation) as the two calls one after the other.  When no
 * sequence completes a quantization group with these tokens -- all but one decode step in
 * group_size -- the whole step is ONE launch: the attention kernel copies the new rows from
 * k_new / v_new into the fp16 ring itself before it reads the ring; otherwise the append's
 * launches come first.  k_new, v_new must stay valid until the call has run on the stream.  n_new == 0: the
 * attention alone.  Errors: those of the two calls; on an error nothing has been enqueued and
 * seq_len_host is unchanged, except that an error of the attention after a separate append
 * leaves the tokens appended.
 */
int32_t tkv_quant_decode(const tkv_quant_desc* desc, tkv_quant_cache* cache, const void* k_new,
                         const void* v_new, int32_t n_new, const int32_t* n_valid_host, const void* q,
                         void* out, float sm_scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * tkv_quant_attn_decode for callers that cannot allocate or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as tkv_quant_attn_decode, but the split-K partials and arrival
 * counters live in a fixed device array inside the library image
 * (TKV_STATIC_MAX_HEADS * 4 + TKV_STATIC_PARTS_BYTES bytes on every GPU the library runs on,
 * held until the process ends).  The call allocates nothing and frees nothing.
 * Limits: batch * n_kv_heads (twice that for groups of more than 4 query heads) <=
 * TKV_STATIC_MAX_HEADS and the launch's partials
 * (batch * n_q_heads * chunks * 528 bytes; chunks is about compute units / (batch * n_kv_heads),
 * at most 64) must fit in TKV_STATIC_PARTS_BYTES, else TKV_E_WORKSPACE and nothing is enqueued.
 * Batch 1 to 64 with 32 query heads fits at every context length.
 * The device that owns `stream` and the buffers must be the calling thread's current device.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or host threads) race with each other and give wrong results; calls on one stream
 * are safe.  The first call on a device looks the array up (no allocation).
 */
#define TKV_STATIC_MAX_HEADS 4096
#define TKV_STATIC_PARTS_BYTES (4u << 20)
int32_t tkv_quant_attn_decode_static(const tkv_quant_desc* desc, const tkv_quant_cache* cache, const void* q,
                                     void* out, float sm_scale, void* stream);

/* ---------------------------------------------------------------------------------
 * Sparsity-friendly layers
 * ------------------------------------------------------------------------------- */

typedef struct {
  uint32_t struct_size; /* sizeof(tkv_sparse_desc)                                        */
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;     /* 128                                                            */
  int32_t n_channels;   /* d_s: critical channels kept on the GPU; 16, 12 or 8 (Sec. 5.1
                           runs 8 and 12)                                                 */
  int32_t top_k;        /* n_topk: tokens fetched per KV head, 1..4096                    */
  int32_t n_sink;       /* first tokens always resident; with n_window this is n_local    */
  int32_t n_window;     /* newest tokens always resident; 1..1024                         */
  int32_t capacity;     /* max tokens per sequence                                        */
  int32_t batch;
} tkv_sparse_desc;

typedef struct {
  void* key_summary;     /* fp16 [B][Hkv][capacity][d_s]: channels channel_idx of every key */
  int32_t* channel_idx;  /* int32 [B][Hkv][d_s] ascending, an input                          */
  void* kv_host;         /* PINNED HOST fp16 [B][Hkv][capacity][2][128]: K row then V row     */
  void* kv_local;        /* fp16 [B][Hkv][n_sink + n_window][2][128]: token t < n_sink at
                            slot t, any other token at slot n_sink + t mod n_window          */
  int32_t* seq_len_host; /* HOST int32 [B]                                                   */
} tkv_sparse_cache;

/* Bytes of key_summary, channel_idx, kv_host, kv_local; workspace bytes for
 * tkv_sparse_estimate_topk and tkv_sparse_gather_attn (the larger of the two). */
int32_t tkv_sparse_cache_sizes(const tkv_sparse_desc* desc, size_t bytes_out[4], size_t* workspace_bytes);

/*
 * Eq. 2 for a sparsity-friendly layer: k_new, v_new fp16 [B][n_new][Hkv][128] (device)
 * are written to the host cache, their critical channels to key_summary and the rows
 * that belong to sinks/window to kv_local.  seq_len_host[b] += n_new.
 */
int32_t tkv_sparse_append(const tkv_sparse_desc* desc, tkv_sparse_cache* cache, const void* k_new,
                          const void* v_new, int32_t n_new, void* stream);
/* Padded-batch form, as tkv_quantize_append_ragged. */
int32_t tkv_sparse_append_ragged(const tkv_sparse_desc* desc, tkv_sparse_cache* cache, const void* k_new,
                                 const void* v_new, int32_t n_new, const int32_t* n_valid_host, void* stream);

/*
 * Stage 2 of Sec. 4.2: approximate scores from the critical query channels and the
 * critical key cache, then Top-K.  For KV head h and candidate token
 * t in [n_sink, N - n_window):
 *     a_j  = (((p_0 + p_1) + p_2) + ... ),  p_i = f32(q_j[c_i]) * f32(summary[t][i]),
 *     S(t) = ((a_0 + a_1) + ...) over the group's query heads j ascending, + 0.0f,
 * all float32, products exact.  The k = min(top_k, #candidates) tokens with the
 * largest S (ties: lower index first) are written to topk_idx [B][Hkv][top_k] in
 * ASCENDING token order, padded with -1; topk_count [B][Hkv] gets k.
 * Scores must be finite.
 * workspace: at least the size tkv_sparse_cache_sizes reports, ZERO-FILLED by the caller
 * before its first use (it holds histograms and counters that every call leaves zero
 * again); concurrent calls need separate workspaces.
 * The tokens are split over about one workgroup per compute unit that `stream` may use
 * (all of them, or those of its compute-unit mask); the result does not depend on it.
 */
int32_t tkv_sparse_estimate_topk(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache, const void* q,
                                 int32_t* topk_idx, int32_t* topk_count, void* workspace,
                                 size_t workspace_bytes, void* stream);

/*
 * A decode step's tkv_sparse_append_ragged and tkv_sparse_estimate_topk in one call (and
 * one launch fewer): the n_new <= min(8, n_window) new tokens are appended by the scoring
 * launch itself (they are newer than every Top-K candidate, so the scores do not depend on
 * them).  Same results as the two calls.  seq_len_host[b] += n_valid on success.
 */
int32_t tkv_sparse_append_estimate_topk(const tkv_sparse_desc* desc, tkv_sparse_cache* cache, const void* k_new,
                                        const void* v_new, int32_t n_new, const int32_t* n_valid_host,
                                        const void* q, int32_t* topk_idx, int32_t* topk_count, void* workspace,
                                        size_t workspace_bytes, void* stream);

/*
 * A sparsity-friendly layer's whole decode step in ONE launch: Eq. 2 for the step's new tokens
 * (n_new 0..min(8, n_window); n_new == 0: k_new, v_new, n_valid_host are ignored), Stage 2
 * scoring and Top-K as in tkv_sparse_estimate_topk, fetch of the selected rows from the host
 * cache and exact attention as in tkv_sparse_gather_attn (Sec. 4.2, Sec. 5.1; Eq. 3).  Same
 * topk_idx / topk_count / out as the separate calls (attention within the same tolerance: the
 * order of the float32 sums differs).  This is the form for a decoder, where a layer's
 * calls cannot overlap with anything: the workgroup that finishes a head's selection goes on to
 * fetch that head's rows and attends to them, so no launch boundary and no cross-workgroup
 * hand-off sits between the selection and the transfer that cannot be hidden.
 * Groups of 5 to 8 query heads per KV head: the same call, same results, as two launches
 * (tkv_sparse_append_estimate_topk, then tkv_sparse_gather_attn on this stream); the hint is
 * not used then.
 * The key summary must be token-major (cache->key_summary).  workspace: as for
 * tkv_sparse_estimate_topk.  seq_len_host[b] += n_valid on success.
 * next_key_summary: NULL, or the key summary (device, same descriptor, hence same layout as
 * cache->key_summary) of the layer whose tkv_sparse_decode is the next call on this stream - in a
 * decoder the next sparsity-friendly layer; a key summary does not depend on its layer's query.
 * The workgroups that are through with the selection read their own share of it once, while the
 * heads' last workgroups wait for the host link and HBM is idle: the next launch finds the rows
 * in the memory-side cache (about 1 us per call at 131072 tokens).  A hint: it is only read, and
 * no result depends on it.
 */
int32_t tkv_sparse_decode(const tkv_sparse_desc* desc, tkv_sparse_cache* cache, const void* k_new,
                          const void* v_new, int32_t n_new, const int32_t* n_valid_host, const void* q,
                          int32_t* topk_idx, int32_t* topk_count, void* out, float sm_scale,
                          const void* next_key_summary, void* workspace, size_t workspace_bytes,
                          void* stream);

/*
 * Fetch of the Top-K tokens from the host cache (Sec. 4.2; the one transfer that
 * cannot be hidden) and exact attention (Eq. 3) of every query head over
 * sinks [0, n_sink) U selected U window [N - n_window, N) (Sec. 5.1: n_local + n_topk).
 * staging: fp16 [B][Hkv][top_k][2][128] device buffer the rows are gathered into.
 * Two different streams: the gather kernel runs on gather_stream after everything
 * already enqueued on compute_stream (which produced topk_idx); attention runs on
 * compute_stream after the gather.  The same stream twice: nothing could overlap, so one
 * kernel fetches the rows from the host cache and attends to them; `staging` is then
 * left untouched (its contents are unspecified).  out: fp16 [B][Hq][128].
 */
int32_t tkv_sparse_gather_attn(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache, const void* q,
                               const int32_t* topk_idx, const int32_t* topk_count, void* out,
                               float sm_scale, void* staging, void* workspace, size_t workspace_bytes,
                               void* gather_stream, void* compute_stream);

/* The two halves of tkv_sparse_gather_attn as separate calls (for pipelining the
 * gather of one layer under other layers' compute, and for timing the link alone).
 * The attention calls use the same workspace as tkv_sparse_estimate_topk, with the same
 * rule: zero-filled before its first use, left consistent by every call. */
int32_t tkv_sparse_gather(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache, const int32_t* topk_idx,
                          const int32_t* topk_count, void* staging, void* stream);
int32_t tkv_sparse_attn(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache, const void* q,
                        const int32_t* topk_count, const void* staging, void* out, float sm_scale,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------
 * Stage 1 of the dynamic retrieval (Sec. 4.2, Fig. 4): critical channels re-estimated
 * every step (Eq. 10) and the critical key cache fetched for them.  Optional: a layer
 * whose channel list is fixed only needs the calls above.
 * ------------------------------------------------------------------------------- */

typedef struct {
  float* k_absmax; /* device fp32 [B][Hkv][128]: max over cached tokens of |K[t][c]| (the
                      second factor of Eq. 10); ZERO before the first append               */
  void* keys_cm;   /* fp16 [B][Hkv][128][capacity], channel-major copy of all keys: pinned
                      host memory (the paper's CPU pool; fetched per step with
                      tkv_sparse_prefetch_keys) or device memory (resident; read in place
                      by tkv_sparse_estimate_topk_cm with rows_per_head = 128)             */
} tkv_sparse_stage1;

/* Bytes of k_absmax and keys_cm. */
int32_t tkv_sparse_stage1_sizes(const tkv_sparse_desc* desc, size_t bytes_out[2]);

/*
 * Cache update of the Stage 1 buffers for the tokens k_new fp16 [B][n_new][Hkv][128]
 * (device) that tkv_sparse_append[_ragged] is about to append: call it BEFORE that
 * append, with the same k_new / n_new / n_valid_host (it reads seq_len_host and leaves
 * it unchanged).  keys_cm receives the transposed rows, k_absmax the running maxima.
 * capacity must be a multiple of 8.
 */
int32_t tkv_sparse_stage1_append(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache,
                                 const tkv_sparse_stage1* stage1, const void* k_new, int32_t n_new,
                                 const int32_t* n_valid_host, void* stream);

/*
 * Eq. 10 per KV head: s_i = (((|q_0,i| + |q_1,i|) + ...) over the group's query heads)
 * * k_absmax[i], every operation one float32 operation; the d_s channels with the
 * largest s (ties: lower channel first) are written to channel_idx_out int32
 * [B][Hkv][d_s] (device) in ASCENDING order.  q_hat: fp16 [B][Hq][128] (device), the
 * query predicted for this layer one layer early (App. B) or the query itself.
 */
int32_t tkv_sparse_select_channels(const tkv_sparse_desc* desc, const tkv_sparse_stage1* stage1,
                                   const void* q_hat, int32_t* channel_idx_out, void* stream);

/*
 * Fetch of the critical key cache (Sec. 4.2, "prefetch"): rows channel_idx[b][h][i] of
 * keys_cm, tokens [0, seq_len), into keys_out fp16 [B][Hkv][d_s][capacity] (device;
 * the caller alternates two such buffers to overlap the fetch for the next layer with
 * this layer's compute).  Bound by the host link when keys_cm is host memory:
 * Hkv * d_s * N * 2 bytes per call.
 */
int32_t tkv_sparse_prefetch_keys(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache,
                                 const tkv_sparse_stage1* stage1, const int32_t* channel_idx, void* keys_out,
                                 void* stream);

/*
 * tkv_sparse_estimate_topk over a channel-major critical key cache: same scores, same
 * selection, same outputs and workspace rules.  keys_cm: device fp16
 * [B][Hkv][rows_per_head][capacity]; rows_per_head = d_s: row i holds channel
 * channel_idx[b][h][i] (what tkv_sparse_prefetch_keys wrote); rows_per_head = 128: row c
 * holds channel c (a resident tkv_sparse_stage1.keys_cm), of which only the listed d_s
 * rows are read.  cache->key_summary is not used.  capacity must be a multiple of 8.
 */
int32_t tkv_sparse_estimate_topk_cm(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache, const void* q,
                                    const int32_t* channel_idx, const void* keys_cm, int32_t rows_per_head,
                                    int32_t* topk_idx, int32_t* topk_count, void* workspace,
                                    size_t workspace_bytes, void* stream);

/*
 * Stage 1 and Stage 2 in one call for RESIDENT channel-major keys (stage1->keys_cm in device
 * memory): Eq. 10 as in tkv_sparse_select_channels (list also written to channel_idx_out),
 * then scoring and Top-K as in tkv_sparse_estimate_topk_cm with rows_per_head = 128.  Nothing
 * crosses the host link.  TKV_E_INVAL if keys_cm is not device memory.
 */
int32_t tkv_sparse_select_estimate_topk(const tkv_sparse_desc* desc, const tkv_sparse_cache* cache,
                                        const tkv_sparse_stage1* stage1, const void* q_hat, const void* q,
                                        int32_t* channel_idx_out, int32_t* topk_idx, int32_t* topk_count,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * tkv_sparse_append_ragged that also keeps the Stage 1 buffers up to date (stage1 may be
 * NULL: then it is tkv_sparse_append_ragged).  Replaces the pair tkv_sparse_stage1_append +
 * tkv_sparse_append_ragged; a decode step's single token costs one launch.
 */
int32_t tkv_sparse_append_dynamic(const tkv_sparse_desc* desc, tkv_sparse_cache* cache,
                                  const tkv_sparse_stage1* stage1, const void* k_new, const void* v_new,
                                  int32_t n_new, const int32_t* n_valid_host, void* stream);

/* ---------------------------------------------------------------------------------
 * Offline identification (Sec. 4.1): which layers are quantization-friendly
 * ------------------------------------------------------------------------------- */

typedef struct {
  uint32_t struct_size; /* sizeof(tkv_pref_desc)                                          */
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;     /* 128                                                            */
  int32_t n_q;          /* most recent query vectors of the prompt used per head (Eq. 6);
                           a multiple of 16, at most 256                                  */
  int32_t top_k;        /* k of Eq. 7, 1..4096                                            */
  int32_t capacity;     /* largest prompt length n                                        */
  int32_t batch;
} tkv_pref_desc;

/* Workspace bytes of tkv_dense_preference: n_q * Hq rows, each with room for
 * min(capacity, 32 * top_k) candidate logits and capacity / 32 partial maxima. */
int32_t tkv_dense_preference_sizes(const tkv_pref_desc* desc, size_t* workspace_bytes);

/*
 * Dense preference score of one layer, Eq. 6-8, per query head:
 *     A = softmax(q_last K^T * sm_scale) row by row over all n keys (Eq. 6 as printed: no
 *     mask), P = n_q - sum over the rows of their top_k largest entries (Eq. 7, 8).
 * q_last: fp16 [B][n_q][Hq][128] (device), the n_q most recent query vectors of the prompt;
 * k: fp16 [B][n][Hkv][128] (device), the prompt's keys (the layout of the append calls);
 * query head j reads KV head j / (Hq/Hkv), any group size.  p_out: float32 [B][Hq] (device).
 * sm_scale > 0 (TKV_E_INVAL otherwise).
 * Logits are float32 (fp16 products accumulated in float32) and are never written to memory:
 * they are computed twice, once for a per-row lower bound of the top_k-th largest logit and
 * once for the softmax denominator and the logits above that bound, among which the top_k
 * largest are then selected exactly; the mass of a row's top_k entries does not depend on how
 * ties are broken.  The result is the same bit for bit from call to call.  workspace:
 * ZERO-FILLED before its first use, left consistent by every call; concurrent calls need
 * separate workspaces.  Sequences of a batch are processed one after the other.
 */
int32_t tkv_dense_preference(const tkv_pref_desc* desc, const void* q_last, const void* k, int32_t n,
                             float sm_scale, float* p_out, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * Eq. 9 on the host.  The layer's score is read as the mean over its heads of P / n_q (the
 * average attention mass outside the top_k keys; Sec. 5.1 uses tau = 0.2); p_heads_host:
 * HOST float32 [n_heads].  Returns 1 (quantization-friendly: score > tau), 0
 * (sparsity-friendly) or a negative tkv_status; the score itself goes to *layer_score_out
 * unless that is NULL.
 */
int32_t tkv_classify_layer(const float* p_heads_host, int32_t n_heads, int32_t n_q, float tau,
                           float* layer_score_out);

#ifdef __cplusplus
}
#endif
#endif /* TKV_H */
