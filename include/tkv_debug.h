/*
 * tkv - test, tuning and measurement hooks.  Not part of the method's interface
 * (tkv.h); a product caller never needs them.
 */
#ifndef TKV_DEBUG_H
#define TKV_DEBUG_H

#include "tkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Test and tuning hook (process-wide; the two settings are atomics, a call that runs
 * concurrently with the change may see either value): kernel_choice 0 = matrix-core
 * kernel, which also covers the fp16 tail (default), 1 = shape-generic
 * reference kernel for everything.  By default the split-K launch aims at one workgroup per
 * compute unit that the stream may use (all of them, or those of its compute-unit mask);
 * target_blocks > 0 fixes the number of workgroups instead, -1 returns to the default, 0
 * keeps the current setting (the launch uses at most 64 chunks per (sequence, KV head)
 * unless target_blocks asks for more than that). */
int32_t tkv_debug_quant_attn_config(int32_t kernel_choice, int32_t target_blocks);

/* Measurement aid (not part of the method): one plain read sweep over `bytes` bytes of
 * device memory at `src` (both multiples of 16), 16-byte loads, n_workgroups workgroups of
 * 256 lanes (1 to 65536).  `sink`: NULL or a device buffer of n_workgroups 32-bit words
 * (almost never written; it only keeps the loads alive).  The benchmark times it over as
 * many bytes as a tkv_quant_attn_decode call reads: what a kernel that does nothing but
 * stream that volume takes on the same machine, launch included. */
int32_t tkv_debug_read_sweep(const void* src, size_t bytes, void* sink, int32_t n_workgroups, void* stream);

/* Test aid: which parts of the workspaces may hold anything between calls.
 * Quantized layers: bytes [0, *scratch_bytes) of the tkv_quant_attn_decode workspace are scratch
 * (split-K partials, fully rewritten by every call before they are read); the rest holds the
 * arrival counters, which must be zero before the first call and are left zero by every call.
 * Sparse layers: region_offsets[0..6] are the byte offsets of: score keys (dense preference
 * score only), candidate lists, histograms (dense preference score only), control words
 * (arrival counters), list lengths, attention partials, end.  The histograms and control words
 * must be zero before the first call and are left zero; everything else is scratch. */
int32_t tkv_debug_quant_workspace(const tkv_quant_desc* desc, size_t* scratch_bytes);
int32_t tkv_debug_sparse_workspace(const tkv_sparse_desc* desc, size_t region_offsets[7]);

#ifdef __cplusplus
}
#endif
#endif /* TKV_DEBUG_H */
