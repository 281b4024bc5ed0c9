// Shared device/host helpers of the gfx950 turn-resumption library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "symph.h"

namespace symph {

constexpr int kWave = 64;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

inline int elem_bytes_of(int32_t dtype) { return dtype == SYMPH_BF16 ? 2 : (dtype == SYMPH_FP32 ? 4 : 0); }

inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Host-side checks every entry point shares. Returns SYMPH_OK or the status to hand back.
int32_t validate_cache(const symph_kv_cache* c);

// Launchers (defined next to their kernels).
int32_t launch_kv_migrate(bool pack, const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                          const int32_t* d_table, int32_t table_stride, const int32_t* d_prefix_lens,
                          const int32_t* d_tail_begin, const int64_t* d_offsets, int32_t n_sessions,
                          int64_t total_tokens, void* d_buf, int64_t buf_bytes, hipStream_t stream,
                          const int64_t* d_chunk_rows = nullptr, bool batch_layer_major = false);
int32_t launch_kv_append(const symph_kv_cache* cache, int32_t layer, const void* d_k_new, const void* d_v_new,
                         const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens, const int32_t* d_table,
                         int32_t table_stride, int32_t n_sessions, int32_t total_new_tokens, hipStream_t stream);
int32_t launch_device_copy(void* d_dst, const void* d_src, int64_t bytes, hipStream_t stream);
int32_t launch_mfma_reference(int32_t iters, int64_t* h_flops, void* d_sink, hipStream_t stream);

struct AttnArgs {
  const void* k_layer;  // K pool of the chosen layer
  const void* v_layer;
  int64_t block_stride;  // elements
  int32_t n_blocks, block_size, n_kv_heads, n_q_heads, head_dim, dtype;
  const void* q;
  const void* k_new;
  const void* v_new;
  void* out;
  const int32_t* cu_new_lens;
  const int32_t* prefix_lens;
  const int32_t* table;
  int32_t table_stride, n_sessions, total_new_tokens, max_new_len, max_prefix_len;
  float scale;
  void* workspace;
  int64_t workspace_bytes;
  const symph_attn_tuning* tuning;  // null: defaults
  bool fit_workspace;               // the workspace has a fixed size: cut the work list so that it is enough
};
int32_t launch_prefill_attn(const AttnArgs& a, hipStream_t stream);
int64_t prefill_attn_workspace_bytes(const symph_kv_cache* cache, int32_t n_sessions, int32_t n_q_heads,
                                     int32_t total_new_tokens, int32_t max_new_len, int32_t max_prefix_len,
                                     const symph_attn_tuning* tuning);
// Validation and argument marshalling shared by the attention entry points (defined with them).
int32_t prefill_attn_entry(const symph_kv_cache* cache, int32_t layer, const void* d_q, const void* d_k_new,
                           const void* d_v_new, void* d_out, const int32_t* d_cu_new_lens,
                           const int32_t* d_prefix_lens, const int32_t* d_block_table, int32_t table_stride,
                           int32_t n_sessions, int32_t n_q_heads, int32_t total_new_tokens, int32_t max_new_len,
                           int32_t max_prefix_len, float scale, void* d_workspace, int64_t workspace_bytes,
                           void* stream, const symph_attn_tuning* tuning, bool fit_workspace);
// Number of ints at the start of the attention workspace that hold counts and flags, and the index of the flags.
constexpr int kAttnHdrInts = 8;
constexpr int kAttnHdrFlags = 7;

}  // namespace symph
