/*
 * symph.h - C ABI of the MI355X (gfx950) turn-resumption library.
 *
 * The operations behind resuming a conversation turn in Symphony (arxiv 2412.16434): a session's K,V cache is
 * moved between GPUs / memory tiers ahead of the next request (Sec. 3.2 "Symphony Node Manager", Sec. 3.3
 * "Hierarchical memory management", "cooperative memory management"), and the new turn then attends to that
 * cached prefix instead of recomputing it (Sec. 2.1 attention definition and "KV Cache", Sec. 2.4 swap vs.
 * recompute).
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers; everything else is passed by value.
 *   - The caller owns every buffer.  The library allocates no memory (symph_debug_check_tables aside) and keeps no
 *     state between calls (it reads no environment variable either: what can be tuned is an explicit argument);
 *     calls may be issued concurrently on different streams as long as the memory they write does not overlap.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work and return
 *     without synchronising; device arrays must stay valid until the stream has executed the work.
 *   - Return value: SYMPH_OK or a negative symph_status.  Nothing aborts or throws across the ABI.  Host-visible
 *     arguments are validated before anything is launched.  Contents of device arrays (block ids, lengths) are
 *     the caller's contract; kernels additionally never touch memory through a block id outside [0, n_blocks) or for
 *     a token beyond the buffer: pack / unpack / append skip such rows, attention reads a row of zeros for them (the
 *     key then has score 0 and value 0 in every kernel of the attention path).
 *
 * Layouts ("element" = one value of cache dtype: bf16 = 2 bytes, fp32 = 4 bytes)
 *   paged cache   K pool and V pool.  Element (layer l, block b, slot o, kv-head g, dim c) of K lives at
 *                 k_base + l*layer_stride + b*block_stride + (o*n_kv_heads + g)*head_dim + c   (elements),
 *                 same for V from v_base.  A block holds block_size consecutive tokens of one session.
 *   block table   int32 [n_sessions][table_stride]; token t of session s is in block table[s][t / block_size],
 *                 slot t % block_size.  Entries past ceil(P_s / block_size) are ignored.
 *   migration buffer   session-major, then layer, then K before V, then token, head, dim; exactly P_s tokens
 *                 per session, no padding.  Row (s, l, kv, t) starts at element
 *                 (off[s]*2*L + (2*l + kv)*P_s + t) * n_kv_heads*head_dim,  off = exclusive prefix sum of P.
 *                 Layer l of a session is thus one contiguous chunk that can be shipped or consumed first
 *                 (Sec. 3.3: layer-wise asynchronous reads/writes, lower layers first).
 *   q, out        [T][n_q_heads][head_dim];  k_new, v_new  [T][n_kv_heads][head_dim];  T = sum of new-turn
 *                 lengths; session s owns rows cu_new_lens[s] .. cu_new_lens[s+1]-1.
 */
#ifndef SYMPH_H_
#define SYMPH_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SYMPH_OK = 0,
  SYMPH_EINVAL = -1,       /* null pointer, non-positive shape, inconsistent sizes, bad scale */
  SYMPH_EUNSUPPORTED = -2, /* shape / dtype / alignment the kernels do not cover */
  SYMPH_ELAUNCH = -3,      /* the HIP runtime refused the launch or copy */
  SYMPH_EWORKSPACE = -4,   /* workspace or buffer smaller than required */
  SYMPH_ENOMEM = -5        /* host memory exhausted (only the stateful host objects of symph_pool.h allocate) */
} symph_status;

typedef enum { SYMPH_BF16 = 0, SYMPH_FP32 = 1 } symph_dtype;

/* A paged K,V cache owned by the caller (device memory). Strides are in elements. */
typedef struct {
  void* k_base;          /* device: K pool, layer 0, block 0 */
  void* v_base;          /* device: V pool, layer 0, block 0 */
  int64_t layer_stride;  /* elements between consecutive layers of one pool */
  int64_t block_stride;  /* elements between consecutive blocks; >= block_size*n_kv_heads*head_dim */
  int32_t n_layers;
  int32_t n_blocks;      /* blocks per layer pool; block ids are 0 .. n_blocks-1 */
  int32_t block_size;    /* tokens per block */
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t dtype;         /* symph_dtype */
} symph_kv_cache;

/* Bytes of the migration buffer for total_tokens cached tokens: total_tokens * 2 * L * n_kv_heads * head_dim *
 * elem_bytes.  (Llama-3.1-70B shape at 32768 tokens gives 10 GiB, the figure in Sec. 1.)  Negative on bad input. */
int64_t symph_kv_buffer_bytes(const symph_kv_cache* cache, int64_t total_tokens);

/*
 * Gather: copy the cached K,V of every listed session, all layers, out of its scattered blocks into the
 * migration buffer (Sec. 3.2: the node manager serves K,V fetch requests from peers and moves caches between
 * tiers; Sec. 3.5: data is not changed - the copy is bit-exact).
 *   d_block_table [n_sessions][table_stride] int32, d_prefix_lens [n_sessions] int32,
 *   d_buf_token_offsets [n_sessions+1] int64 (exclusive prefix sum of prefix lengths),
 *   total_tokens = host copy of d_buf_token_offsets[n_sessions] (sizes the grid without a device read-back),
 *   d_buf: device, buf_bytes >= symph_kv_buffer_bytes(cache, total_tokens), 16-byte aligned.  Any address the
 *   device can reach will do: pinned host memory that the runtime maps for the device (hipHostMalloc) makes the
 *   kernel write (pack) or read (unpack) it over the host link, without a staging copy in device memory.
 * Reads only slots of valid tokens (never the unused tail of a partially filled last block); a block id may
 * appear in several sessions.  n_sessions == 0 or total_tokens == 0 is SYMPH_OK with no launch.
 * Needs row bytes (n_kv_heads*head_dim*elem) to be a multiple of 4 and strides/pointers aligned to
 * min(16, largest power of two dividing the row bytes).
 */
int32_t symph_kv_pack(const symph_kv_cache* cache, const int32_t* d_block_table, int32_t table_stride,
                      const int32_t* d_prefix_lens, const int64_t* d_buf_token_offsets, int32_t n_sessions,
                      int64_t total_tokens, void* d_buf, int64_t buf_bytes, void* stream);

/*
 * Scatter: the inverse of symph_kv_pack through a destination block table taken from the free list (Sec. 3.3:
 * the node manager greedily fills free GPU memory with arriving caches; Sec. 3.4 cases 1-3).  Writes only the
 * slots of valid tokens; every other byte of the pools is left untouched.  A block id listed twice in the
 * destination table has two writers and the result for that block is undefined.
 */
int32_t symph_kv_unpack(const symph_kv_cache* cache, const int32_t* d_dst_block_table, int32_t table_stride,
                        const int32_t* d_prefix_lens, const int64_t* d_buf_token_offsets, int32_t n_sessions,
                        int64_t total_tokens, const void* d_buf, int64_t buf_bytes, void* stream);

/*
 * The same gather / scatter restricted to layers layer_begin .. layer_end-1 (Sec. 3.3: K,V are read and written layer
 * by layer, asynchronously, so that a transfer overlaps the inference of the layers already there; a request whose
 * lower layers have arrived can start).  The buffer keeps the layout and size of the whole cache: layer l of session
 * s is the contiguous chunk of 2 * P_s rows (K then V) that starts (offsets[s] * 2 * L + 2 * l * P_s) rows into the
 * buffer.  Buffer bytes of other layers (pack) and pool bytes of other layers (unpack) are not touched.
 * 0 <= layer_begin <= layer_end <= n_layers; an empty range is SYMPH_OK with no launch.  Everything else as above.
 */
int32_t symph_kv_pack_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                             const int32_t* d_block_table, int32_t table_stride, const int32_t* d_prefix_lens,
                             const int64_t* d_buf_token_offsets, int32_t n_sessions, int64_t total_tokens, void* d_buf,
                             int64_t buf_bytes, void* stream);
int32_t symph_kv_unpack_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                               const int32_t* d_dst_block_table, int32_t table_stride, const int32_t* d_prefix_lens,
                               const int64_t* d_buf_token_offsets, int32_t n_sessions, int64_t total_tokens,
                               const void* d_buf, int64_t buf_bytes, void* stream);

/*
 * The same layer-range gather / scatter with a BATCH-LEVEL LAYER-MAJOR buffer (Sec. 3.3, layer-wise reads and writes):
 * layer first, then session, then K before V, then token, i.e. row (l, s, K|V, t) starts
 *   (l * 2 * total_tokens + offsets[s] * 2 + kv * P_s + t)
 * rows into the buffer.  Layer l of the WHOLE batch is then one contiguous piece of 2 * total_tokens rows, which one
 * copy moves (symph_stage_batch_layers_*), where the session-major buffer above needs one copy per session and layer.
 * Same size as the session-major buffer, same rows in another order; everything else as for symph_kv_pack_layers.
 */
int32_t symph_kv_pack_batch_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                   const int32_t* d_block_table, int32_t table_stride, const int32_t* d_prefix_lens,
                                   const int64_t* d_buf_token_offsets, int32_t n_sessions, int64_t total_tokens,
                                   void* d_buf, int64_t buf_bytes, void* stream);
int32_t symph_kv_unpack_batch_layers(const symph_kv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                     const int32_t* d_dst_block_table, int32_t table_stride,
                                     const int32_t* d_prefix_lens, const int64_t* d_buf_token_offsets,
                                     int32_t n_sessions, int64_t total_tokens, const void* d_buf, int64_t buf_bytes,
                                     void* stream);

/*
 * Write-back of what a turn added (Sec. 3.3: the slower memory tiers are kept up to date with newly generated K,V, so
 * that the fast tier can be purged at any time): the gather / scatter for tokens d_tail_begin[s] .. d_prefix_lens[s]-1
 * of every session only, all layers.  The buffer has the layout of a migration buffer for sessions of the tail lengths
 * T_s = prefix_lens[s] - tail_begin[s]: d_tail_offsets[S+1] (device, int64) is the exclusive prefix sum of the T_s,
 * total_tail_tokens its last entry (host copy), row (s, l, K|V, i) holds token tail_begin[s] + i, buf_bytes >=
 * symph_kv_buffer_bytes(cache, total_tail_tokens).  Appending, per (session, layer, K|V), a tail's rows to the rows
 * packed when the session had tail_begin[s] tokens gives the rows of a whole pack at the present length.  A session
 * with tail_begin[s] outside [0, prefix_lens[s]] is skipped.  Everything else as for symph_kv_pack / symph_kv_unpack.
 */
int32_t symph_kv_pack_tail(const symph_kv_cache* cache, const int32_t* d_block_table, int32_t table_stride,
                           const int32_t* d_prefix_lens, const int32_t* d_tail_begin, const int64_t* d_tail_offsets,
                           int32_t n_sessions, int64_t total_tail_tokens, void* d_buf, int64_t buf_bytes, void* stream);
int32_t symph_kv_unpack_tail(const symph_kv_cache* cache, const int32_t* d_dst_block_table, int32_t table_stride,
                             const int32_t* d_prefix_lens, const int32_t* d_tail_begin, const int64_t* d_tail_offsets,
                             int32_t n_sessions, int64_t total_tail_tokens, const void* d_buf, int64_t buf_bytes,
                             void* stream);

/*
 * Append: write the new turn's K,V rows of one layer into the paged cache behind each session's prefix, so that the
 * next turn or decode step finds them there (Sec. 2.1 "KV Cache": the keys and values of every processed token are
 * kept; Sec. 3.3: the K,V a request produced join its session's cache).  Token i of session s has position P_s + i:
 * block d_block_table[s][(P_s + i) / block_size], slot (P_s + i) % block_size; the table must list blocks for
 * positions up to P_s + N_s - 1 (the caller takes them from its free list).  d_k_new / d_v_new
 * [total_new_tokens][n_kv_heads][head_dim] in the cache dtype, d_cu_new_lens [n_sessions+1] int32.  Rows whose block
 * id lies outside the cache are skipped; no other byte of the pools changes; the lengths are the caller's to update.
 */
int32_t symph_kv_append(const symph_kv_cache* cache, int32_t layer, const void* d_k_new, const void* d_v_new,
                        const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens, const int32_t* d_block_table,
                        int32_t table_stride, int32_t n_sessions, int32_t total_new_tokens, void* stream);

/*
 * Prefix-cached prefill attention for one layer (Sec. 2.1: A_h = softmax(Q_h K_h^T * scale), y = concat_h A_h V_h;
 * "KV Cache": a token attends to all prior tokens).  For session s, query head h, new token i:
 *   out[cu[s]+i][h][:] = sum_j softmax_j(scale * <q, k_j>) v_j,   j over the P_s cached keys (paged, kv-head
 *   h / (n_q_heads / n_kv_heads)) followed by new keys 0..i of k_new / v_new (causal, self included).
 * The new turn's K,V are NOT yet in the paged cache; they are passed as k_new / v_new.
 *   layer: which layer of `cache` holds the prefix.  q/k_new/v_new/out have the cache dtype.
 *   d_cu_new_lens [n_sessions+1] int32, d_prefix_lens [n_sessions] int32, d_block_table as above.
 *   total_new_tokens = T, max_new_len >= max N_s, max_prefix_len >= max P_s (host copies).  total_new_tokens and
 *   n_sessions size the grids and the work list; max_prefix_len is only checked against the table width; max_new_len
 *   only chooses kernels: a batch with max_new_len * (n_q_heads / n_kv_heads) <= 32 is a decode step and its short
 *   turns run in a kernel that streams K,V with one wave per kv-head.  Neither of the two is relied on for memory safety: a
 *   session longer than stated is still computed, and computed correctly (a turn with more new tokens than stated is
 *   not a short turn for the device-side scheduler and goes through the general kernel), only not at the best speed.
 *   scale > 0 and finite (fp32).  d_workspace: device scratch of at least
 *   symph_prefix_prefill_attn_workspace_bytes(...) bytes, 256-byte aligned (may be NULL when that is 0).
 * Arithmetic: bf16 inputs, fp32 accumulation on MFMA, fp32 online softmax, probabilities rounded to bf16 before
 * the P*V product, output rounded to nearest even; fp32 inputs are computed in fp32 throughout.
 * Supported: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads.  Sessions with N_s == 0 produce no rows;
 * P_s == 0 is a plain causal prefill.  The matrix-core kernels cover bf16, head_dim 128, group sizes 1, 2, 4, 8, 16 and
 * block sizes that are powers of two >= 16; every other supported shape (fp32, head_dim 64, other group sizes, smaller
 * blocks) runs a plain kernel with one wave per query row: correct, not tuned, and its workspace query returns 0.
 */
int32_t symph_prefix_prefill_attn(const symph_kv_cache* cache, int32_t layer, const void* d_q, const void* d_k_new,
                                  const void* d_v_new, void* d_out, const int32_t* d_cu_new_lens,
                                  const int32_t* d_prefix_lens, const int32_t* d_block_table, int32_t table_stride,
                                  int32_t n_sessions, int32_t n_q_heads, int32_t total_new_tokens,
                                  int32_t max_new_len, int32_t max_prefix_len, float scale, void* d_workspace,
                                  int64_t workspace_bytes, void* stream);

/* Scratch bytes symph_prefix_prefill_attn needs for these host-side bounds (the same values as in the call; 0 is
 * possible).  Negative on bad input. */
int64_t symph_prefix_prefill_attn_workspace_bytes(const symph_kv_cache* cache, int32_t n_sessions, int32_t n_q_heads,
                                                  int32_t total_new_tokens, int32_t max_new_len,
                                                  int32_t max_prefix_len);

/*
 * How the attention call cuts a ragged batch into workgroup-sized pieces (Sec. 2.2: prefill is compute-bound, decode
 * memory-bound, and one batch mixes both).  A field that is 0 keeps its default, so a zeroed struct, or a null
 * pointer, is the default behaviour; the values do not change what is computed, only how the work is divided.
 */
typedef struct {
  int32_t slots;       /* workgroups resident on the GPU at once, which the work list is balanced for (default 512) */
  int32_t c_min;       /* shortest piece of a (session, query tile) unit that is split, in 64-key tiles (default 8) */
  int32_t coarse;      /* > 0 (default): with at least two units per slot only the longest units are split; < 0: every
                          unit is cut so that there are about two pieces per slot */
  int32_t decode;      /* > 0 (default): decode steps (see max_new_len above) take the streaming kernel; < 0: never */
  int32_t decode_wgs;  /* that kernel runs 4 * decode_wgs waves, one per (key range, kv-head): 4 * decode_wgs /
                          n_kv_heads ranges (default 512: with 8 kv-heads one 8-wave workgroup per compute unit) */
  int32_t reserved[3]; /* 0 */
} symph_attn_tuning;

/* The same two calls with explicit tuning values.  The workspace query and the call must be given the same values: a
 * call whose workspace is smaller than its own values require returns SYMPH_EWORKSPACE. */
int32_t symph_prefix_prefill_attn_tuned(const symph_kv_cache* cache, int32_t layer, const void* d_q,
                                        const void* d_k_new, const void* d_v_new, void* d_out,
                                        const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens,
                                        const int32_t* d_block_table, int32_t table_stride, int32_t n_sessions,
                                        int32_t n_q_heads, int32_t total_new_tokens, int32_t max_new_len,
                                        int32_t max_prefix_len, float scale, void* d_workspace,
                                        int64_t workspace_bytes, void* stream, const symph_attn_tuning* tuning);
int64_t symph_prefix_prefill_attn_workspace_bytes_tuned(const symph_kv_cache* cache, int32_t n_sessions,
                                                        int32_t n_q_heads, int32_t total_new_tokens,
                                                        int32_t max_new_len, int32_t max_prefix_len,
                                                        const symph_attn_tuning* tuning);

/*
 * symph_prefix_prefill_attn for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace, same kernels,
 * same results up to the order in which partial results are combined; the scratch memory is a fixed array of 64 MiB
 * inside the library's device code (one copy per GPU the library is used on, held until the process ends).  The
 * call allocates nothing and frees nothing.  The first call on a device looks the array's address up once
 * (hipGetSymbolAddress) - make that call outside a graph capture.  The work list is cut so that its partial results
 * fit the array (fewer, longer pieces than the workspace version may choose); a batch whose list of query tiles alone
 * needs more than the array (about a million query tiles) returns SYMPH_EWORKSPACE and nothing is launched.  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams) race and must be
 * serialised by the caller; calls on one stream, or ordered by events, are fine, and nothing has to be cleared between
 * them.
 */
int32_t symph_prefix_prefill_attn_static(const symph_kv_cache* cache, int32_t layer, const void* d_q,
                                         const void* d_k_new, const void* d_v_new, void* d_out,
                                         const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens,
                                         const int32_t* d_block_table, int32_t table_stride, int32_t n_sessions,
                                         int32_t n_q_heads, int32_t total_new_tokens, int32_t max_new_len,
                                         int32_t max_prefix_len, float scale, void* stream);

/*
 * What the device-side scheduler of the last attention call on `d_workspace` reported (a debugging aid like
 * symph_debug_check_tables: it copies one word to the host and synchronises `stream`).  *h_flags: bit 0 - a unit that
 * should have been split was left whole because the workspace has no room for its pieces (slower, still correct; it
 * cannot happen with a workspace of the queried size); bit 1 - the lengths on the device describe more query tiles
 * than total_new_tokens and n_sessions allow, and the work beyond that bound was NOT done (the caller broke the
 * contract on d_cu_new_lens).  0 for shapes that need no workspace.
 */
#define SYMPH_ATTN_FLAG_UNSPLIT 1
#define SYMPH_ATTN_FLAG_DROPPED 2
int32_t symph_debug_attn_flags(const void* d_workspace, void* stream, int32_t* h_flags);

/*
 * Host staging on a side stream (Sec. 2.4 "Swap": K,V swapped to host memory; Sec. 3.3: asynchronous reads and
 * writes so transfers overlap inference).  symph_stage_to_host orders a device->host copy of `bytes` bytes
 * after everything already enqueued on `producer_stream` (typically the pack) and runs it on `side_stream`;
 * symph_stage_to_device runs a host->device copy on `side_stream` and makes `consumer_stream` (typically the
 * unpack) wait for it.  h_pinned must be pinned host memory (hipHostMalloc) for the copy to be asynchronous.
 * `event` is a caller-created hipEvent_t (as void*) used for the ordering; it may be reused once the streams
 * have passed it.  side_stream must differ from the other stream.
 */
int32_t symph_stage_to_host(void* h_pinned, const void* d_buf, int64_t bytes, void* producer_stream,
                            void* side_stream, void* event);
int32_t symph_stage_to_device(void* d_buf, const void* h_pinned, int64_t bytes, void* consumer_stream,
                              void* side_stream, void* event);

/*
 * Host staging of ONE layer of every listed session (Sec. 3.3, layer-wise transfers): the n_sessions chunks of
 * layer `layer` (see symph_kv_pack_layers for where they lie; same offsets in the pinned host buffer, which has the
 * size of the whole device buffer) are copied on `side_stream`.  to_host: after everything already enqueued on
 * `producer_stream`; to_device: `consumer_stream` then waits for the copies.  h_prefix_lens [n_sessions] and
 * h_buf_token_offsets [n_sessions+1] are HOST arrays (the copies are sized on the host); row_bytes =
 * n_kv_heads * head_dim * elem_bytes of the cache.  `event` as above.
 */
int32_t symph_stage_layer_to_host(void* h_pinned, const void* d_buf, const symph_kv_cache* cache, int32_t layer,
                                  const int32_t* h_prefix_lens, const int64_t* h_buf_token_offsets,
                                  int32_t n_sessions, void* producer_stream, void* side_stream, void* event);
int32_t symph_stage_layer_to_device(void* d_buf, const void* h_pinned, const symph_kv_cache* cache, int32_t layer,
                                    const int32_t* h_prefix_lens, const int64_t* h_buf_token_offsets,
                                    int32_t n_sessions, void* consumer_stream, void* side_stream, void* event);

/*
 * Host staging of layers layer_begin .. layer_end-1 of a batch-level layer-major buffer (see symph_kv_pack_batch_layers):
 * ONE copy of (layer_end - layer_begin) * 2 * total_tokens rows on `side_stream`, at the same offset in the device
 * buffer and in the pinned host buffer (which has the size of the whole device buffer); ordering through `event` as for
 * symph_stage_to_host / symph_stage_to_device.  Needs no host copies of the lengths.
 */
int32_t symph_stage_batch_layers_to_host(void* h_pinned, const void* d_buf, const symph_kv_cache* cache,
                                         int32_t layer_begin, int32_t layer_end, int64_t total_tokens,
                                         void* producer_stream, void* side_stream, void* event);
int32_t symph_stage_batch_layers_to_device(void* d_buf, const void* h_pinned, const symph_kv_cache* cache,
                                           int32_t layer_begin, int32_t layer_end, int64_t total_tokens,
                                           void* consumer_stream, void* side_stream, void* event);

/*
 * Unit-wise gather / scatter (Sec. 3.3, priority-based K,V cache: single layers of sessions are moved in, lower layers
 * first, and given up, later layers first; with several announced sessions only their lower layers may be resident).
 * `slots` describes ONE pool of slots with n_layers = 1: a slot holds a block of any layer (symph_pool.h hands the
 * slot numbers out).  Unit u is one layer of one session: d_unit_lens[u] tokens, token t in slot
 * d_unit_table[u][t / block_size]; in the buffer its K rows start at row d_unit_chunk_rows[u] (rows of
 * n_kv_heads * head_dim elements) and its V rows d_unit_lens[u] rows later, which is where layer l of session s lies
 * in a whole migration buffer when chunk_rows = off[s] * 2 * L + 2 * l * P_s.  d_unit_token_offsets [n_units+1] is the
 * exclusive prefix sum of the lengths (it splits the launch's work), total_unit_tokens its last entry.  All units go
 * in one launch; nothing else in the pool or the buffer is touched; a unit whose chunk would pass buf_bytes, or with a
 * negative chunk row, is skipped.  buf_bytes is the size of the whole buffer (at least 2 * total_unit_tokens rows).
 */
int32_t symph_kv_pack_units(const symph_kv_cache* slots, const int32_t* d_unit_table, int32_t table_stride,
                            const int32_t* d_unit_lens, const int64_t* d_unit_token_offsets,
                            const int64_t* d_unit_chunk_rows, int32_t n_units, int64_t total_unit_tokens, void* d_buf,
                            int64_t buf_bytes, void* stream);
int32_t symph_kv_unpack_units(const symph_kv_cache* slots, const int32_t* d_unit_table, int32_t table_stride,
                              const int32_t* d_unit_lens, const int64_t* d_unit_token_offsets,
                              const int64_t* d_unit_chunk_rows, int32_t n_units, int64_t total_unit_tokens,
                              const void* d_buf, int64_t buf_bytes, void* stream);

/*
 * Optional check of what the kernels take on trust (the caller's contract on device-resident contents): every length
 * is >= 0 and fits its table row, every block id a session uses lies in [0, n_blocks), and - for a destination table
 * (is_destination != 0: unpack, append) - no block is named twice, within a session or across sessions.  d_lens are
 * the lengths the table has to cover (prefix lengths, or prefix + new-turn lengths before an append).  A debugging
 * aid, unlike every other entry point: it copies both arrays to host memory it allocates for the call and
 * synchronises `stream`.  Returns SYMPH_OK, or SYMPH_EINVAL with the first offending session in *h_first_bad_session
 * (may be null; -1 if the arguments themselves were invalid).
 */
int32_t symph_debug_check_tables(const symph_kv_cache* cache, const int32_t* d_block_table, int32_t table_stride,
                                 const int32_t* d_lens, int32_t n_sessions, int32_t is_destination, void* stream,
                                 int32_t* h_first_bad_session);

/* Plain contiguous device copy with the same 16-byte-per-lane access shape as pack / unpack: the practical
 * HBM ceiling the migration kernels are compared with, and the known-size kernel used to calibrate hardware
 * traffic counters.  bytes must be a multiple of 16, pointers 16-byte aligned. */
int32_t symph_device_copy(void* d_dst, const void* d_src, int64_t bytes, void* stream);

/* Matrix-core reference: every wave of 2 * (number of CUs) workgroups of four waves runs 32 * iters dependent-free
 * v_mfma_f32_32x32x16_bf16 instructions on registers (no memory traffic), the bf16 dense rate the attention kernel is
 * compared with next to the published peak.  *h_flops (host, may be null) receives the floating-point operations of
 * one launch; d_sink is a device word the kernel may write (it never does for finite inputs).  The caller times it. */
int32_t symph_mfma_reference(int32_t iters, int64_t* h_flops, void* d_sink, void* stream);

const char* symph_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* SYMPH_H_ */
