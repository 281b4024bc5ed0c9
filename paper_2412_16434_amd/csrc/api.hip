// extern "C" entry points: host-side validation, then launches. No allocation, no global state.
#include "common.h"

#include <new>
#include <vector>

namespace symph {

int32_t validate_cache(const symph_kv_cache* c) {
  if (!c) return SYMPH_EINVAL;
  if (!c->k_base || !c->v_base) return SYMPH_EINVAL;
  if (c->n_layers <= 0 || c->n_blocks <= 0 || c->block_size <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0)
    return SYMPH_EINVAL;
  if (elem_bytes_of(c->dtype) == 0) return SYMPH_EUNSUPPORTED;
  const int64_t block_elems = (int64_t)c->block_size * c->n_kv_heads * c->head_dim;
  if (c->block_stride < block_elems) return SYMPH_EINVAL;
  if (c->n_layers > 1 && c->layer_stride <= 0) return SYMPH_EINVAL;
  return SYMPH_OK;
}

static int32_t migrate(bool pack, const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                       const int32_t* d_table, int32_t table_stride, const int32_t* d_prefix_lens,
                       const int64_t* d_offsets, int32_t n_sessions, int64_t total_tokens, void* d_buf,
                       int64_t buf_bytes, void* stream, const int32_t* d_tail_begin = nullptr,
                       const int64_t* d_chunk_rows = nullptr, bool batch_layer_major = false) {
  int32_t rc = validate_cache(cache);
  if (rc != SYMPH_OK) return rc;
  if (n_sessions < 0 || total_tokens < 0 || table_stride < 0 || buf_bytes < 0) return SYMPH_EINVAL;
  if (layer_begin < 0 || layer_end > cache->n_layers || layer_begin > layer_end) return SYMPH_EINVAL;
  if (n_sessions == 0 || total_tokens == 0 || layer_begin == layer_end) return SYMPH_OK;
  if (!d_table || !d_prefix_lens || !d_offsets || !d_buf || table_stride == 0) return SYMPH_EINVAL;
  const int64_t need = symph_kv_buffer_bytes(cache, total_tokens);
  if (need < 0) return SYMPH_EINVAL;
  if (buf_bytes < need) return SYMPH_EWORKSPACE;
  return launch_kv_migrate(pack, cache, layer_begin, layer_end, d_table, table_stride, d_prefix_lens, d_tail_begin,
                           d_offsets, n_sessions, total_tokens, d_buf, buf_bytes, (hipStream_t)stream, d_chunk_rows,
                           batch_layer_major);
}

// Units (single layers of sessions) between one pool of slots and chunks placed anywhere in the buffer.
static int32_t migrate_units(bool pack, const symph_kv_cache* slots, const int32_t* d_table, int32_t table_stride,
                             const int32_t* d_unit_lens, const int64_t* d_unit_token_offsets,
                             const int64_t* d_unit_chunk_rows, int32_t n_units, int64_t total_unit_tokens, void* d_buf,
                             int64_t buf_bytes, void* stream) {
  if (!slots) return SYMPH_EINVAL;
  if (slots->n_layers != 1) return SYMPH_EINVAL;  // the slot pool has no layer axis: a slot holds a block of any layer
  if (n_units > 0 && total_unit_tokens > 0 && !d_unit_chunk_rows) return SYMPH_EINVAL;
  return migrate(pack, slots, 0, 1, d_table, table_stride, d_unit_lens, d_unit_token_offsets, n_units,
                 total_unit_tokens, d_buf, buf_bytes, stream, nullptr, d_unit_chunk_rows);
}

// The chunk of one layer of one session in the migration buffer (bytes): 2 * P rows of K then V.
static inline void layer_chunk(const symph_kv_cache* c, int32_t layer, int64_t offset_s, int32_t P, int64_t* begin,
                               int64_t* bytes) {
  const int64_t row_bytes = (int64_t)c->n_kv_heads * c->head_dim * elem_bytes_of(c->dtype);
  *begin = (offset_s * 2 * c->n_layers + (int64_t)2 * layer * P) * row_bytes;
  *bytes = (int64_t)2 * P * row_bytes;
}

static int32_t stage_layer(bool to_host, void* dst, const void* src, const symph_kv_cache* cache, int32_t layer,
                           const int32_t* h_prefix_lens, const int64_t* h_offsets, int32_t n_sessions,
                           void* other_stream, void* side_stream, void* event) {
  int32_t rc = validate_cache(cache);
  if (rc != SYMPH_OK) return rc;
  if (layer < 0 || layer >= cache->n_layers || n_sessions < 0) return SYMPH_EINVAL;
  if (n_sessions == 0) return SYMPH_OK;
  if (!dst || !src || !h_prefix_lens || !h_offsets || !event || side_stream == other_stream) return SYMPH_EINVAL;
  for (int32_t s = 0; s < n_sessions; ++s)
    if (h_prefix_lens[s] < 0 || h_offsets[s] < 0 || h_offsets[s + 1] - h_offsets[s] < h_prefix_lens[s]) return SYMPH_EINVAL;
  if (to_host) {  // the copies follow what the producer has enqueued so far
    if (hipEventRecord((hipEvent_t)event, (hipStream_t)other_stream) != hipSuccess) return SYMPH_ELAUNCH;
    if (hipStreamWaitEvent((hipStream_t)side_stream, (hipEvent_t)event, 0) != hipSuccess) return SYMPH_ELAUNCH;
  }
  for (int32_t s = 0; s < n_sessions; ++s) {
    int64_t begin, bytes;
    layer_chunk(cache, layer, h_offsets[s], h_prefix_lens[s], &begin, &bytes);
    if (bytes == 0) continue;
    if (hipMemcpyAsync((char*)dst + begin, (const char*)src + begin, (size_t)bytes,
                       to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, (hipStream_t)side_stream) != hipSuccess)
      return SYMPH_ELAUNCH;
  }
  if (!to_host) {  // the consumer waits for the copies
    if (hipEventRecord((hipEvent_t)event, (hipStream_t)side_stream) != hipSuccess) return SYMPH_ELAUNCH;
    if (hipStreamWaitEvent((hipStream_t)other_stream, (hipEvent_t)event, 0) != hipSuccess) return SYMPH_ELAUNCH;
  }
  return SYMPH_OK;
}

}  // namespace symph

using namespace symph;

extern "C" {

int64_t symph_kv_buffer_bytes(const symph_kv_cache* cache, int64_t total_tokens) {
  if (!cache || total_tokens < 0) return -1;
  const int eb = elem_bytes_of(cache->dtype);
  if (eb == 0 || cache->n_layers <= 0 || cache->n_kv_heads <= 0 || cache->head_dim <= 0) return -1;
  return total_tokens * 2 * (int64_t)cache->n_layers * cache->n_kv_heads * cache->head_dim * eb;
}

int32_t symph_kv_pack(const symph_kv_cache* cache, const int32_t* d_block_table, int32_t table_stride,
                      const int32_t* d_prefix_lens, const int64_t* d_buf_token_offsets, int32_t n_sessions,
                      int64_t total_tokens, void* d_buf, int64_t buf_bytes, void* stream) {
  if (!cache) return SYMPH_EINVAL;
  return migrate(true, cache, 0, cache->n_layers, d_block_table, table_stride, d_prefix_lens, d_buf_token_offsets,
                 n_sessions, total_tokens, d_buf, buf_bytes, stream);
}

int32_t symph_kv_pack_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                             const int32_t* d_block_table, int32_t table_stride, const int32_t* d_prefix_lens,
                             const int64_t* d_buf_token_offsets, int32_t n_sessions, int64_t total_tokens, void* d_buf,
                             int64_t buf_bytes, void* stream) {
  return migrate(true, cache, layer_begin, layer_end, d_block_table, table_stride, d_prefix_lens, d_buf_token_offsets,
                 n_sessions, total_tokens, d_buf, buf_bytes, stream);
}

int32_t symph_kv_pack_batch_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                   const int32_t* d_block_table, int32_t table_stride, const int32_t* d_prefix_lens,
                                   const int64_t* d_buf_token_offsets, int32_t n_sessions, int64_t total_tokens,
                                   void* d_buf, int64_t buf_bytes, void* stream) {
  return migrate(true, cache, layer_begin, layer_end, d_block_table, table_stride, d_prefix_lens, d_buf_token_offsets,
                 n_sessions, total_tokens, d_buf, buf_bytes, stream, nullptr, nullptr, true);
}

int32_t symph_kv_unpack_batch_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                     const int32_t* d_dst_block_table, int32_t table_stride,
                                     const int32_t* d_prefix_lens, const int64_t* d_buf_token_offsets,
                                     int32_t n_sessions, int64_t total_tokens, const void* d_buf, int64_t buf_bytes,
                                     void* stream) {
  return migrate(false, cache, layer_begin, layer_end, d_dst_block_table, table_stride, d_prefix_lens,
                 d_buf_token_offsets, n_sessions, total_tokens, const_cast<void*>(d_buf), buf_bytes, stream, nullptr,
                 nullptr, true);
}

// One contiguous copy of layers layer_begin .. layer_end-1 of a batch-level layer-major buffer.
static int32_t stage_batch_layers(bool to_host, void* dst, const void* src, const symph_kv_cache* cache,
                                  int32_t layer_begin, int32_t layer_end, int64_t total_tokens, void* other_stream,
                                  void* side_stream, void* event) {
  int32_t rc = validate_cache(cache);
  if (rc != SYMPH_OK) return rc;
  if (layer_begin < 0 || layer_end > cache->n_layers || layer_begin > layer_end || total_tokens < 0) return SYMPH_EINVAL;
  if (layer_begin == layer_end || total_tokens == 0) return SYMPH_OK;
  if (!dst || !src || !event || side_stream == other_stream) return SYMPH_EINVAL;
  const int64_t layer_bytes = 2 * total_tokens * (int64_t)cache->n_kv_heads * cache->head_dim * elem_bytes_of(cache->dtype);
  const int64_t begin = layer_begin * layer_bytes, bytes = (layer_end - layer_begin) * layer_bytes;
  if (to_host) {  // the copy follows what the producer has enqueued so far
    if (hipEventRecord((hipEvent_t)event, (hipStream_t)other_stream) != hipSuccess) return SYMPH_ELAUNCH;
    if (hipStreamWaitEvent((hipStream_t)side_stream, (hipEvent_t)event, 0) != hipSuccess) return SYMPH_ELAUNCH;
  }
  if (hipMemcpyAsync((char*)dst + begin, (const char*)src + begin, (size_t)bytes,
                     to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, (hipStream_t)side_stream) != hipSuccess)
    return SYMPH_ELAUNCH;
  if (!to_host) {  // the consumer waits for the copy
    if (hipEventRecord((hipEvent_t)event, (hipStream_t)side_stream) != hipSuccess) return SYMPH_ELAUNCH;
    if (hipStreamWaitEvent((hipStream_t)other_stream, (hipEvent_t)event, 0) != hipSuccess) return SYMPH_ELAUNCH;
  }
  return SYMPH_OK;
}

int32_t symph_stage_batch_layers_to_host(void* h_pinned, const void* d_buf, const symph_kv_cache* cache,
                                         int32_t layer_begin, int32_t layer_end, int64_t total_tokens,
                                         void* producer_stream, void* side_stream, void* event) {
  return stage_batch_layers(true, h_pinned, d_buf, cache, layer_begin, layer_end, total_tokens, producer_stream,
                            side_stream, event);
}

int32_t symph_stage_batch_layers_to_device(void* d_buf, const void* h_pinned, const symph_kv_cache* cache,
                                           int32_t layer_begin, int32_t layer_end, int64_t total_tokens,
                                           void* consumer_stream, void* side_stream, void* event) {
  return stage_batch_layers(false, d_buf, h_pinned, cache, layer_begin, layer_end, total_tokens, consumer_stream,
                            side_stream, event);
}

int32_t symph_kv_pack_tail(const symph_kv_cache* cache, const int32_t* d_block_table, int32_t table_stride,
                           const int32_t* d_prefix_lens, const int32_t* d_tail_begin, const int64_t* d_tail_offsets,
                           int32_t n_sessions, int64_t total_tail_tokens, void* d_buf, int64_t buf_bytes, void* stream) {
  if (!cache) return SYMPH_EINVAL;
  if (n_sessions > 0 && total_tail_tokens > 0 && !d_tail_begin) return SYMPH_EINVAL;
  return migrate(true, cache, 0, cache->n_layers, d_block_table, table_stride, d_prefix_lens, d_tail_offsets,
                 n_sessions, total_tail_tokens, d_buf, buf_bytes, stream, d_tail_begin);
}

int32_t symph_kv_unpack_tail(const symph_kv_cache* cache, const int32_t* d_dst_block_table, int32_t table_stride,
                             const int32_t* d_prefix_lens, const int32_t* d_tail_begin, const int64_t* d_tail_offsets,
                             int32_t n_sessions, int64_t total_tail_tokens, const void* d_buf, int64_t buf_bytes,
                             void* stream) {
  if (!cache) return SYMPH_EINVAL;
  if (n_sessions > 0 && total_tail_tokens > 0 && !d_tail_begin) return SYMPH_EINVAL;
  return migrate(false, cache, 0, cache->n_layers, d_dst_block_table, table_stride, d_prefix_lens, d_tail_offsets,
                 n_sessions, total_tail_tokens, const_cast<void*>(d_buf), buf_bytes, stream, d_tail_begin);
}

int32_t symph_kv_pack_units(const symph_kv_cache* slots, const int32_t* d_unit_table, int32_t table_stride,
                            const int32_t* d_unit_lens, const int64_t* d_unit_token_offsets,
                            const int64_t* d_unit_chunk_rows, int32_t n_units, int64_t total_unit_tokens, void* d_buf,
                            int64_t buf_bytes, void* stream) {
  return migrate_units(true, slots, d_unit_table, table_stride, d_unit_lens, d_unit_token_offsets, d_unit_chunk_rows,
                       n_units, total_unit_tokens, d_buf, buf_bytes, stream);
}

int32_t symph_kv_unpack_units(const symph_kv_cache* slots, const int32_t* d_unit_table, int32_t table_stride,
                              const int32_t* d_unit_lens, const int64_t* d_unit_token_offsets,
                              const int64_t* d_unit_chunk_rows, int32_t n_units, int64_t total_unit_tokens,
                              const void* d_buf, int64_t buf_bytes, void* stream) {
  return migrate_units(false, slots, d_unit_table, table_stride, d_unit_lens, d_unit_token_offsets, d_unit_chunk_rows,
                       n_units, total_unit_tokens, const_cast<void*>(d_buf), buf_bytes, stream);
}

int32_t symph_kv_unpack(const symph_kv_cache* cache, const int32_t* d_dst_block_table, int32_t table_stride,
                        const int32_t* d_prefix_lens, const int64_t* d_buf_token_offsets, int32_t n_sessions,
                        int64_t total_tokens, const void* d_buf, int64_t buf_bytes, void* stream) {
  if (!cache) return SYMPH_EINVAL;
  return migrate(false, cache, 0, cache->n_layers, d_dst_block_table, table_stride, d_prefix_lens,
                 d_buf_token_offsets, n_sessions, total_tokens, const_cast<void*>(d_buf), buf_bytes, stream);
}

int32_t symph_kv_unpack_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                               const int32_t* d_dst_block_table, int32_t table_stride, const int32_t* d_prefix_lens,
                               const int64_t* d_buf_token_offsets, int32_t n_sessions, int64_t total_tokens,
                               const void* d_buf, int64_t buf_bytes, void* stream) {
  return migrate(false, cache, layer_begin, layer_end, d_dst_block_table, table_stride, d_prefix_lens,
                 d_buf_token_offsets, n_sessions, total_tokens, const_cast<void*>(d_buf), buf_bytes, stream);
}

int32_t symph_kv_append(const symph_kv_cache* cache, int32_t layer, const void* d_k_new, const void* d_v_new,
                        const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens, const int32_t* d_block_table,
                        int32_t table_stride, int32_t n_sessions, int32_t total_new_tokens, void* stream) {
  int32_t rc = validate_cache(cache);
  if (rc != SYMPH_OK) return rc;
  if (layer < 0 || layer >= cache->n_layers) return SYMPH_EINVAL;
  if (n_sessions < 0 || total_new_tokens < 0 || table_stride < 0) return SYMPH_EINVAL;
  if (n_sessions == 0 || total_new_tokens == 0) return SYMPH_OK;
  if (!d_k_new || !d_v_new || !d_cu_new_lens || !d_prefix_lens || !d_block_table || table_stride == 0)
    return SYMPH_EINVAL;
  return launch_kv_append(cache, layer, d_k_new, d_v_new, d_cu_new_lens, d_prefix_lens, d_block_table, table_stride,
                          n_sessions, total_new_tokens, (hipStream_t)stream);
}

int64_t symph_prefix_prefill_attn_workspace_bytes_tuned(const symph_kv_cache* cache, int32_t n_sessions,
                                                        int32_t n_q_heads, int32_t total_new_tokens,
                                                        int32_t max_new_len, int32_t max_prefix_len,
                                                        const symph_attn_tuning* tuning) {
  if (!cache || n_sessions < 0 || n_q_heads <= 0 || total_new_tokens < 0 || max_new_len < 0 || max_prefix_len < 0)
    return -1;
  if (cache->n_kv_heads <= 0) return -1;
  return prefill_attn_workspace_bytes(cache, n_sessions, n_q_heads, total_new_tokens, max_new_len, max_prefix_len,
                                      tuning);
}

int64_t symph_prefix_prefill_attn_workspace_bytes(const symph_kv_cache* cache, int32_t n_sessions, int32_t n_q_heads,
                                                  int32_t total_new_tokens, int32_t max_new_len,
                                                  int32_t max_prefix_len) {
  return symph_prefix_prefill_attn_workspace_bytes_tuned(cache, n_sessions, n_q_heads, total_new_tokens, max_new_len,
                                                         max_prefix_len, nullptr);
}

}  // extern "C"

namespace symph {
// Validation and argument marshalling shared by the attention entry points.
int32_t prefill_attn_entry(const symph_kv_cache* cache, int32_t layer, const void* d_q, const void* d_k_new,
                           const void* d_v_new, void* d_out, const int32_t* d_cu_new_lens,
                           const int32_t* d_prefix_lens, const int32_t* d_block_table, int32_t table_stride,
                           int32_t n_sessions, int32_t n_q_heads, int32_t total_new_tokens, int32_t max_new_len,
                           int32_t max_prefix_len, float scale, void* d_workspace, int64_t workspace_bytes,
                           void* stream, const symph_attn_tuning* tuning, bool fit_workspace) {
  int32_t rc = validate_cache(cache);
  if (rc != SYMPH_OK) return rc;
  if (layer < 0 || layer >= cache->n_layers) return SYMPH_EINVAL;
  if (n_sessions < 0 || total_new_tokens < 0 || max_new_len < 0 || max_prefix_len < 0 || table_stride < 0 ||
      workspace_bytes < 0)
    return SYMPH_EINVAL;
  if (n_q_heads <= 0 || n_q_heads % cache->n_kv_heads != 0) return SYMPH_EINVAL;
  if (!(scale > 0.0f) || !(scale < INFINITY)) return SYMPH_EINVAL;
  if (max_new_len > total_new_tokens) return SYMPH_EINVAL;
  if (n_sessions == 0 || total_new_tokens == 0) return SYMPH_OK;
  if (!d_q || !d_k_new || !d_v_new || !d_out || !d_cu_new_lens || !d_prefix_lens) return SYMPH_EINVAL;
  if (max_prefix_len > 0 && (!d_block_table || table_stride == 0)) return SYMPH_EINVAL;
  if (max_prefix_len > 0 && (int64_t)table_stride * cache->block_size < max_prefix_len) return SYMPH_EINVAL;
  if (cache->head_dim != 64 && cache->head_dim != 128) return SYMPH_EUNSUPPORTED;
  if (tuning && (tuning->slots < 0 || tuning->c_min < 0 || tuning->decode_wgs < 0)) return SYMPH_EINVAL;
  const int64_t need = prefill_attn_workspace_bytes(cache, n_sessions, n_q_heads, total_new_tokens, max_new_len,
                                                    max_prefix_len, tuning);
  if (need > 0 && !fit_workspace && (!d_workspace || workspace_bytes < need)) return SYMPH_EWORKSPACE;

  const int eb = elem_bytes_of(cache->dtype);
  AttnArgs a;
  a.k_layer = (const char*)cache->k_base + (int64_t)layer * cache->layer_stride * eb;
  a.v_layer = (const char*)cache->v_base + (int64_t)layer * cache->layer_stride * eb;
  a.block_stride = cache->block_stride;
  a.n_blocks = cache->n_blocks;
  a.block_size = cache->block_size;
  a.n_kv_heads = cache->n_kv_heads;
  a.n_q_heads = n_q_heads;
  a.head_dim = cache->head_dim;
  a.dtype = cache->dtype;
  a.q = d_q;
  a.k_new = d_k_new;
  a.v_new = d_v_new;
  a.out = d_out;
  a.cu_new_lens = d_cu_new_lens;
  a.prefix_lens = d_prefix_lens;
  a.table = d_block_table;
  a.table_stride = table_stride;
  a.n_sessions = n_sessions;
  a.total_new_tokens = total_new_tokens;
  a.max_new_len = max_new_len;
  a.max_prefix_len = max_prefix_len;
  a.scale = scale;
  a.workspace = d_workspace;
  a.workspace_bytes = workspace_bytes;
  a.tuning = tuning;
  a.fit_workspace = fit_workspace;
  return launch_prefill_attn(a, (hipStream_t)stream);
}
}  // namespace symph

extern "C" {

int32_t symph_prefix_prefill_attn_tuned(const symph_kv_cache* cache, int32_t layer, const void* d_q,
                                        const void* d_k_new, const void* d_v_new, void* d_out,
                                        const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens,
                                        const int32_t* d_block_table, int32_t table_stride, int32_t n_sessions,
                                        int32_t n_q_heads, int32_t total_new_tokens, int32_t max_new_len,
                                        int32_t max_prefix_len, float scale, void* d_workspace,
                                        int64_t workspace_bytes, void* stream, const symph_attn_tuning* tuning) {
  return prefill_attn_entry(cache, layer, d_q, d_k_new, d_v_new, d_out, d_cu_new_lens, d_prefix_lens, d_block_table,
                            table_stride, n_sessions, n_q_heads, total_new_tokens, max_new_len, max_prefix_len, scale,
                            d_workspace, workspace_bytes, stream, tuning, false);
}

int32_t symph_prefix_prefill_attn(const symph_kv_cache* cache, int32_t layer, const void* d_q, const void* d_k_new,
                                  const void* d_v_new, void* d_out, const int32_t* d_cu_new_lens,
                                  const int32_t* d_prefix_lens, const int32_t* d_block_table, int32_t table_stride,
                                  int32_t n_sessions, int32_t n_q_heads, int32_t total_new_tokens,
                                  int32_t max_new_len, int32_t max_prefix_len, float scale, void* d_workspace,
                                  int64_t workspace_bytes, void* stream) {
  return prefill_attn_entry(cache, layer, d_q, d_k_new, d_v_new, d_out, d_cu_new_lens, d_prefix_lens, d_block_table,
                            table_stride, n_sessions, n_q_heads, total_new_tokens, max_new_len, max_prefix_len, scale,
                            d_workspace, workspace_bytes, stream, nullptr, false);
}

int32_t symph_debug_attn_flags(const void* d_workspace, void* stream, int32_t* h_flags) {
  if (!h_flags) return SYMPH_EINVAL;
  *h_flags = 0;
  if (!d_workspace) return SYMPH_OK;  // a shape without a workspace has no scheduler
  int32_t hdr[kAttnHdrInts];
  if (hipMemcpyAsync(hdr, d_workspace, sizeof(hdr), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess ||
      hipStreamSynchronize((hipStream_t)stream) != hipSuccess)
    return SYMPH_ELAUNCH;
  *h_flags = hdr[kAttnHdrFlags];
  return SYMPH_OK;
}

int32_t symph_stage_to_host(void* h_pinned, const void* d_buf, int64_t bytes, void* producer_stream,
                            void* side_stream, void* event) {
  if (bytes < 0) return SYMPH_EINVAL;
  if (bytes == 0) return SYMPH_OK;
  if (!h_pinned || !d_buf || !event || side_stream == producer_stream) return SYMPH_EINVAL;
  if (hipEventRecord((hipEvent_t)event, (hipStream_t)producer_stream) != hipSuccess) return SYMPH_ELAUNCH;
  if (hipStreamWaitEvent((hipStream_t)side_stream, (hipEvent_t)event, 0) != hipSuccess) return SYMPH_ELAUNCH;
  if (hipMemcpyAsync(h_pinned, d_buf, (size_t)bytes, hipMemcpyDeviceToHost, (hipStream_t)side_stream) != hipSuccess)
    return SYMPH_ELAUNCH;
  return SYMPH_OK;
}

int32_t symph_stage_to_device(void* d_buf, const void* h_pinned, int64_t bytes, void* consumer_stream,
                              void* side_stream, void* event) {
  if (bytes < 0) return SYMPH_EINVAL;
  if (bytes == 0) return SYMPH_OK;
  if (!h_pinned || !d_buf || !event || side_stream == consumer_stream) return SYMPH_EINVAL;
  if (hipMemcpyAsync(d_buf, h_pinned, (size_t)bytes, hipMemcpyHostToDevice, (hipStream_t)side_stream) != hipSuccess)
    return SYMPH_ELAUNCH;
  if (hipEventRecord((hipEvent_t)event, (hipStream_t)side_stream) != hipSuccess) return SYMPH_ELAUNCH;
  if (hipStreamWaitEvent((hipStream_t)consumer_stream, (hipEvent_t)event, 0) != hipSuccess) return SYMPH_ELAUNCH;
  return SYMPH_OK;
}

int32_t symph_stage_layer_to_host(void* h_pinned, const void* d_buf, const symph_kv_cache* cache, int32_t layer,
                                  const int32_t* h_prefix_lens, const int64_t* h_buf_token_offsets,
                                  int32_t n_sessions, void* producer_stream, void* side_stream, void* event) {
  return stage_layer(true, h_pinned, d_buf, cache, layer, h_prefix_lens, h_buf_token_offsets, n_sessions,
                     producer_stream, side_stream, event);
}

int32_t symph_stage_layer_to_device(void* d_buf, const void* h_pinned, const symph_kv_cache* cache, int32_t layer,
                                    const int32_t* h_prefix_lens, const int64_t* h_buf_token_offsets,
                                    int32_t n_sessions, void* consumer_stream, void* side_stream, void* event) {
  return stage_layer(false, d_buf, h_pinned, cache, layer, h_prefix_lens, h_buf_token_offsets, n_sessions,
                     consumer_stream, side_stream, event);
}

int32_t symph_device_copy(void* d_dst, const void* d_src, int64_t bytes, void* stream) {
  if (bytes < 0) return SYMPH_EINVAL;
  if (bytes == 0) return SYMPH_OK;
  if (!d_dst || !d_src) return SYMPH_EINVAL;
  if ((bytes & 15) || (((uintptr_t)d_dst | (uintptr_t)d_src) & 15)) return SYMPH_EUNSUPPORTED;
  return launch_device_copy(d_dst, d_src, bytes, (hipStream_t)stream);
}

int32_t symph_debug_check_tables(const symph_kv_cache* cache, const int32_t* d_block_table, int32_t table_stride,
                                 const int32_t* d_lens, int32_t n_sessions, int32_t is_destination, void* stream,
                                 int32_t* h_first_bad_session) {
  if (h_first_bad_session) *h_first_bad_session = -1;
  if (!cache || cache->n_blocks <= 0 || cache->block_size <= 0 || n_sessions < 0 || table_stride < 0) return SYMPH_EINVAL;
  if (n_sessions == 0) return SYMPH_OK;
  if (!d_block_table || !d_lens || table_stride == 0) return SYMPH_EINVAL;
  try {
    std::vector<int32_t> lens((size_t)n_sessions), table((size_t)n_sessions * table_stride);
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(lens.data(), d_lens, lens.size() * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipMemcpyAsync(table.data(), d_block_table, table.size() * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
      return SYMPH_ELAUNCH;
    std::vector<uint8_t> taken;
    if (is_destination) taken.assign((size_t)cache->n_blocks, 0);
    for (int32_t s = 0; s < n_sessions; ++s) {
      bool bad = lens[s] < 0;
      const int64_t nb = bad ? 0 : ceil_div64(lens[s], cache->block_size);
      if (nb > table_stride) bad = true;
      for (int64_t j = 0; j < nb && !bad; ++j) {
        const int32_t b = table[(size_t)s * table_stride + j];
        if (b < 0 || b >= cache->n_blocks) {
          bad = true;
        } else if (is_destination) {
          if (taken[b]) bad = true;
          taken[b] = 1;
        }
      }
      if (bad) {
        if (h_first_bad_session) *h_first_bad_session = s;
        return SYMPH_EINVAL;
      }
    }
  } catch (const std::bad_alloc&) {
    return SYMPH_ENOMEM;
  }
  return SYMPH_OK;
}

int32_t symph_mfma_reference(int32_t iters, int64_t* h_flops, void* d_sink, void* stream) {
  if (iters <= 0 || !d_sink) return SYMPH_EINVAL;
  return launch_mfma_reference(iters, h_flops, d_sink, (hipStream_t)stream);
}

const char* symph_status_string(int32_t status) {
  switch (status) {
    case SYMPH_OK: return "ok";
    case SYMPH_EINVAL: return "invalid argument";
    case SYMPH_EUNSUPPORTED: return "unsupported shape, dtype or alignment";
    case SYMPH_ELAUNCH: return "HIP launch or copy failed";
    case SYMPH_EWORKSPACE: return "buffer or workspace too small";
    case SYMPH_ENOMEM: return "out of host memory";
    default: return "unknown status";
  }
}

}  // extern "C"
