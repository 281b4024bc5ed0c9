/*
 * CPU oracle for the turn-resumption path: naive K,V pack / unpack and fp64 softmax attention.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is deliberately plain and slow, shares no code with the HIP library, and
 * may only be called from the test-suite, the smoke check and the benchmark's CPU-baseline leg.
 *
 * What it follows (Symphony, arxiv 2412.16434):
 *   - pack / unpack: the node manager moves a session's K,V cache between memory tiers and between nodes
 *     without changing the data (Sec. 3.2 "Symphony Node Manager", Sec. 3.3 "Hierarchical memory management"
 *     and "cooperative memory management", Sec. 3.5 "Accuracy impact").  The operation therefore has a plain
 *     definition, a permutation copy of bytes, and the functions below are that definition written out.
 *   - attention: Sec. 2.1 "Decoder Only Transformer": A_h = sigma(Q^h K^hT / sqrt(d)), y = concat_h A_h V_h,
 *     with sigma read as the row-wise softmax; Sec. 2.1 "KV Cache": a token needs the keys and values of all
 *     prior tokens, i.e. the new turn's token i sees the whole cached prefix and new tokens 0..i (causal).
 *     Grouped-query attention (query head h uses K,V head floor(h / G)) is the Llama convention; the paper
 *     defines multi-head attention only, which is the G = 1 case.
 *
 * Layouts (all "elements" are of the cache dtype, 2-byte bf16 bit patterns or 4-byte IEEE floats):
 *   K pool and V pool:  element (layer l, block b, slot o, kv-head g, dim c) at
 *                       l*layer_stride + b*block_stride + (o*H_kv + g)*d + c          from k_base / v_base
 *   migration buffer:   session-major, then layer, then K before V, then token, then head, then dim:
 *                       ((off[s]*2L + (2l+kv)*P_s + t) * H_kv + g) * d + c            with off = prefix sum of P
 *   block table:        int32 [S][table_stride]; token t of session s lives in block table[s][t / bs], slot t % bs
 *   q [T][H_q][d], k_new / v_new [T][H_kv][d], T = sum N_s, session s owns rows cu[s] .. cu[s+1]-1
 *
 * Pins (tests/test_oracle_pins.py): closed-form tagged pools, memcpy / transpose special cases, round trips,
 * the paper's cache-size figures, brute-force full-matrix softmax, the cached-prefix == full-recompute
 * invariant, weights summing to one, and closed-form attention cases.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Bytes of a migration buffer holding total_tokens cached tokens: K and V, every layer, no padding. */
int64_t oracle_kv_buffer_bytes(int32_t n_layers, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                               int64_t total_tokens) {
  return total_tokens * 2 * (int64_t)n_layers * n_kv_heads * head_dim * elem_bytes;
}

/* Where one token row (session s, layer l, kv = 0 for K / 1 for V, token t) sits: element offset inside its
 * pool (relative to k_base or v_base) and element offset inside the migration buffer. */
void oracle_kv_locate(int64_t layer_stride, int64_t block_stride, int32_t n_layers, int32_t block_size,
                      int32_t n_kv_heads, int32_t head_dim, const int32_t* table, int32_t table_stride,
                      const int32_t* prefix_lens, const int64_t* offsets, int32_t s, int32_t l, int32_t kv,
                      int32_t t, int64_t* pool_elem, int64_t* buf_elem) {
  const int64_t row = (int64_t)n_kv_heads * head_dim;
  const int64_t b = table[(int64_t)s * table_stride + t / block_size];
  const int64_t o = t % block_size;
  *pool_elem = (int64_t)l * layer_stride + b * block_stride + o * row;
  *buf_elem = (offsets[s] * 2 * n_layers + ((int64_t)2 * l + kv) * prefix_lens[s] + t) * row;
}

/* The whole index function written out as a table: for every row of the migration buffer, in buffer order, the
 * element offset of the row it is a copy of inside its pool, and whether that pool is K (0) or V (1).  A loop over
 * oracle_kv_locate and nothing else; it lets a checker that cannot hold the pools on the host (tens of GiB) compare
 * every row of a buffer, or of a destination pool, against values that are a function of the pool offset.
 * pool_elem_of_row, kv_of_row: offsets[n_sessions] * 2 * n_layers entries each. */
void oracle_kv_row_map(int64_t layer_stride, int64_t block_stride, int32_t n_layers, int32_t block_size,
                       int32_t n_kv_heads, int32_t head_dim, const int32_t* table, int32_t table_stride,
                       const int32_t* prefix_lens, const int64_t* offsets, int32_t n_sessions,
                       int64_t* pool_elem_of_row, uint8_t* kv_of_row) {
  const int64_t row = (int64_t)n_kv_heads * head_dim;
  for (int32_t s = 0; s < n_sessions; ++s)
    for (int32_t l = 0; l < n_layers; ++l)
      for (int32_t kv = 0; kv < 2; ++kv)
        for (int32_t t = 0; t < prefix_lens[s]; ++t) {
          int64_t pe, be;
          oracle_kv_locate(layer_stride, block_stride, n_layers, block_size, n_kv_heads, head_dim, table,
                           table_stride, prefix_lens, offsets, s, l, kv, t, &pe, &be);
          pool_elem_of_row[be / row] = pe;
          kv_of_row[be / row] = (uint8_t)kv;
        }
}

/* Layers layer_begin .. layer_end-1 only: the buffer keeps the layout of the whole cache (Sec. 3.3 moves K,V layer by
 * layer; a layer of a session is one contiguous chunk of the layer-major buffer), everything else is not touched. */
static int kv_copy(int to_buffer, void* k_base, void* v_base, int64_t layer_stride, int64_t block_stride,
                   int32_t n_layers, int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                   const int32_t* table, int32_t table_stride, const int32_t* prefix_lens, const int64_t* offsets,
                   int32_t n_sessions, void* buf, int32_t layer_begin, int32_t layer_end) {
  if (elem_bytes != 2 && elem_bytes != 4) return -1;
  if (layer_begin < 0 || layer_end > n_layers || layer_begin > layer_end) return -1;
  const size_t row_bytes = (size_t)n_kv_heads * head_dim * elem_bytes;
  /* every (s, l) pair touches its own rows of the buffer and its own pool slots, so the pairs are independent */
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int32_t s = 0; s < n_sessions; ++s)
    for (int32_t l = layer_begin; l < layer_end; ++l)
      for (int32_t kv = 0; kv < 2; ++kv)
        for (int32_t t = 0; t < prefix_lens[s]; ++t) {
          int64_t pe, be;
          oracle_kv_locate(layer_stride, block_stride, n_layers, block_size, n_kv_heads, head_dim, table,
                           table_stride, prefix_lens, offsets, s, l, kv, t, &pe, &be);
          char* in_pool = (char*)(kv ? v_base : k_base) + pe * elem_bytes;
          char* in_buf = (char*)buf + be * elem_bytes;
          if (to_buffer)
            memcpy(in_buf, in_pool, row_bytes);
          else
            memcpy(in_pool, in_buf, row_bytes);
        }
  return 0;
}

/* Gather: buffer <- pools.  Reads only slots of valid tokens; writes exactly oracle_kv_buffer_bytes bytes. */
int oracle_kv_pack(const void* k_base, const void* v_base, int64_t layer_stride, int64_t block_stride,
                   int32_t n_layers, int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                   const int32_t* table, int32_t table_stride, const int32_t* prefix_lens, const int64_t* offsets,
                   int32_t n_sessions, void* buf) {
  return kv_copy(1, (void*)k_base, (void*)v_base, layer_stride, block_stride, n_layers, block_size, n_kv_heads,
                 head_dim, elem_bytes, table, table_stride, prefix_lens, offsets, n_sessions, buf, 0, n_layers);
}

/* The gather restricted to layers layer_begin .. layer_end-1 (the rest of the buffer is left as it was). */
int oracle_kv_pack_layers(const void* k_base, const void* v_base, int64_t layer_stride, int64_t block_stride,
                          int32_t n_layers, int32_t block_size, int32_t n_kv_heads, int32_t head_dim,
                          int32_t elem_bytes, const int32_t* table, int32_t table_stride, const int32_t* prefix_lens,
                          const int64_t* offsets, int32_t n_sessions, void* buf, int32_t layer_begin,
                          int32_t layer_end) {
  return kv_copy(1, (void*)k_base, (void*)v_base, layer_stride, block_stride, n_layers, block_size, n_kv_heads,
                 head_dim, elem_bytes, table, table_stride, prefix_lens, offsets, n_sessions, buf, layer_begin,
                 layer_end);
}

/* Scatter: pools <- buffer, through the destination table.  Every pool byte that no valid token owns is left
 * as it was (unlisted blocks and the unused tail slots of a partially filled last block). */
int oracle_kv_unpack(void* k_base, void* v_base, int64_t layer_stride, int64_t block_stride, int32_t n_layers,
                     int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                     const int32_t* table, int32_t table_stride, const int32_t* prefix_lens, const int64_t* offsets,
                     int32_t n_sessions, const void* buf) {
  return kv_copy(0, k_base, v_base, layer_stride, block_stride, n_layers, block_size, n_kv_heads, head_dim,
                 elem_bytes, table, table_stride, prefix_lens, offsets, n_sessions, (void*)buf, 0, n_layers);
}

/* The scatter restricted to layers layer_begin .. layer_end-1 (the other layers of the pools are left as they were). */
int oracle_kv_unpack_layers(void* k_base, void* v_base, int64_t layer_stride, int64_t block_stride, int32_t n_layers,
                            int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                            const int32_t* table, int32_t table_stride, const int32_t* prefix_lens,
                            const int64_t* offsets, int32_t n_sessions, const void* buf, int32_t layer_begin,
                            int32_t layer_end) {
  return kv_copy(0, k_base, v_base, layer_stride, block_stride, n_layers, block_size, n_kv_heads, head_dim,
                 elem_bytes, table, table_stride, prefix_lens, offsets, n_sessions, (void*)buf, layer_begin, layer_end);
}

/* The batch-level layer-major buffer: layer first, then session, then K before V, then token.  Sec. 3.3 reads and
 * writes K,V layer by layer so that a transfer overlaps the inference of the layers that are already there; with the
 * layer outermost, layer l of the WHOLE batch is one contiguous piece of 2 * total rows (total = offsets[n_sessions])
 * that one copy moves.  Row (l, s, kv, t) sits at row l * 2 * total + offsets[s] * 2 + kv * P_s + t of the buffer; the
 * buffer has the size of the session-major one and holds the same rows in another order. */
void oracle_kv_locate_batch_layers(int64_t layer_stride, int64_t block_stride, int32_t block_size, int32_t n_kv_heads,
                                   int32_t head_dim, const int32_t* table, int32_t table_stride,
                                   const int32_t* prefix_lens, const int64_t* offsets, int32_t n_sessions, int32_t s,
                                   int32_t l, int32_t kv, int32_t t, int64_t* pool_elem, int64_t* buf_elem) {
  const int64_t row = (int64_t)n_kv_heads * head_dim;
  const int64_t total = offsets[n_sessions];
  const int64_t b = table[(int64_t)s * table_stride + t / block_size];
  const int64_t o = t % block_size;
  *pool_elem = (int64_t)l * layer_stride + b * block_stride + o * row;
  *buf_elem = ((int64_t)l * 2 * total + offsets[s] * 2 + (int64_t)kv * prefix_lens[s] + t) * row;
}

/* Gather (to_buffer) or scatter of layers layer_begin .. layer_end-1 with the batch-level layer-major buffer. */
int oracle_kv_copy_batch_layers(int to_buffer, void* k_base, void* v_base, int64_t layer_stride, int64_t block_stride,
                                int32_t n_layers, int32_t block_size, int32_t n_kv_heads, int32_t head_dim,
                                int32_t elem_bytes, const int32_t* table, int32_t table_stride,
                                const int32_t* prefix_lens, const int64_t* offsets, int32_t n_sessions, void* buf,
                                int32_t layer_begin, int32_t layer_end) {
  if (elem_bytes != 2 && elem_bytes != 4) return -1;
  if (layer_begin < 0 || layer_end > n_layers || layer_begin > layer_end) return -1;
  const size_t row_bytes = (size_t)n_kv_heads * head_dim * elem_bytes;
  for (int32_t l = layer_begin; l < layer_end; ++l)
    for (int32_t s = 0; s < n_sessions; ++s)
      for (int32_t kv = 0; kv < 2; ++kv)
        for (int32_t t = 0; t < prefix_lens[s]; ++t) {
          int64_t pe, be;
          oracle_kv_locate_batch_layers(layer_stride, block_stride, block_size, n_kv_heads, head_dim, table,
                                        table_stride, prefix_lens, offsets, n_sessions, s, l, kv, t, &pe, &be);
          char* in_pool = (char*)(kv ? v_base : k_base) + pe * elem_bytes;
          char* in_buf = (char*)buf + be * elem_bytes;
          if (to_buffer)
            memcpy(in_buf, in_pool, row_bytes);
          else
            memcpy(in_pool, in_buf, row_bytes);
        }
  return 0;
}

/* Write-back of what a turn added (Sec. 3.3: the slower tiers are kept up to date with newly generated K,V, layer by
 * layer): only tokens tail_begin[s] .. prefix_lens[s]-1 of each session move.  The buffer has the layout of a whole
 * migration buffer for sessions of tail length T_s = prefix_lens[s] - tail_begin[s]: offsets[] counts tail tokens,
 * and row (s, l, kv, i) holds token tail_begin[s] + i.  With tail_begin = 0 this is the whole gather / scatter. */
static int kv_copy_tail(int to_buffer, void* k_base, void* v_base, int64_t layer_stride, int64_t block_stride,
                        int32_t n_layers, int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                        const int32_t* table, int32_t table_stride, const int32_t* prefix_lens,
                        const int32_t* tail_begin, const int64_t* offsets, int32_t n_sessions, void* buf) {
  if (elem_bytes != 2 && elem_bytes != 4) return -1;
  const int64_t row = (int64_t)n_kv_heads * head_dim;
  for (int32_t s = 0; s < n_sessions; ++s)
    if (tail_begin[s] < 0 || tail_begin[s] > prefix_lens[s]) return -1;
  for (int32_t s = 0; s < n_sessions; ++s) {
    const int64_t T = prefix_lens[s] - tail_begin[s];
    for (int32_t l = 0; l < n_layers; ++l)
      for (int32_t kv = 0; kv < 2; ++kv)
        for (int64_t i = 0; i < T; ++i) {
          const int64_t t = tail_begin[s] + i;
          const int64_t b = table[(int64_t)s * table_stride + t / block_size];
          const int64_t pool_elem = (int64_t)l * layer_stride + b * block_stride + (t % block_size) * row;
          const int64_t buf_elem = (offsets[s] * 2 * n_layers + ((int64_t)2 * l + kv) * T + i) * row;
          char* in_pool = (char*)(kv ? v_base : k_base) + pool_elem * elem_bytes;
          char* in_buf = (char*)buf + buf_elem * elem_bytes;
          if (to_buffer)
            memcpy(in_buf, in_pool, (size_t)row * elem_bytes);
          else
            memcpy(in_pool, in_buf, (size_t)row * elem_bytes);
        }
  }
  return 0;
}

int oracle_kv_pack_tail(const void* k_base, const void* v_base, int64_t layer_stride, int64_t block_stride,
                        int32_t n_layers, int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                        const int32_t* table, int32_t table_stride, const int32_t* prefix_lens,
                        const int32_t* tail_begin, const int64_t* offsets, int32_t n_sessions, void* buf) {
  return kv_copy_tail(1, (void*)k_base, (void*)v_base, layer_stride, block_stride, n_layers, block_size, n_kv_heads,
                      head_dim, elem_bytes, table, table_stride, prefix_lens, tail_begin, offsets, n_sessions, buf);
}

int oracle_kv_unpack_tail(void* k_base, void* v_base, int64_t layer_stride, int64_t block_stride, int32_t n_layers,
                          int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes,
                          const int32_t* table, int32_t table_stride, const int32_t* prefix_lens,
                          const int32_t* tail_begin, const int64_t* offsets, int32_t n_sessions, const void* buf) {
  return kv_copy_tail(0, k_base, v_base, layer_stride, block_stride, n_layers, block_size, n_kv_heads, head_dim,
                      elem_bytes, table, table_stride, prefix_lens, tail_begin, offsets, n_sessions, (void*)buf);
}

/* Unit-wise copy (Sec. 3.3, priority-based K,V cache: single layers of sessions are moved in and given up, lower
 * layers first, and with several announced sessions only their lower layers may be resident).  The cache memory is
 * ONE pool of slots, each a block of any layer; unit u is one layer of one session: unit_lens[u] tokens, token t in
 * slot table[u][t / block_size] at position t % block_size, and in the buffer its K rows start at row chunk_rows[u],
 * its V rows unit_lens[u] rows later (where layer l of session s lies in a whole migration buffer:
 * chunk_rows = offsets[s] * 2 * n_layers + 2 * l * P_s).  Nothing else in the pool or the buffer changes. */
static int kv_copy_units(int to_buffer, void* k_base, void* v_base, int64_t block_stride, int32_t block_size,
                         int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes, const int32_t* table,
                         int32_t table_stride, const int32_t* unit_lens, const int64_t* chunk_rows, int32_t n_units,
                         void* buf) {
  if (elem_bytes != 2 && elem_bytes != 4) return -1;
  const int64_t row = (int64_t)n_kv_heads * head_dim;
  for (int32_t u = 0; u < n_units; ++u)
    for (int32_t kv = 0; kv < 2; ++kv)
      for (int64_t t = 0; t < unit_lens[u]; ++t) {
        const int64_t slot = table[(int64_t)u * table_stride + t / block_size];
        const int64_t pool_elem = slot * block_stride + (t % block_size) * row;
        const int64_t buf_elem = (chunk_rows[u] + (int64_t)kv * unit_lens[u] + t) * row;
        char* in_pool = (char*)(kv ? v_base : k_base) + pool_elem * elem_bytes;
        char* in_buf = (char*)buf + buf_elem * elem_bytes;
        if (to_buffer)
          memcpy(in_buf, in_pool, (size_t)row * elem_bytes);
        else
          memcpy(in_pool, in_buf, (size_t)row * elem_bytes);
      }
  return 0;
}

int oracle_kv_pack_units(const void* k_base, const void* v_base, int64_t block_stride, int32_t block_size,
                         int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes, const int32_t* table,
                         int32_t table_stride, const int32_t* unit_lens, const int64_t* chunk_rows, int32_t n_units,
                         void* buf) {
  return kv_copy_units(1, (void*)k_base, (void*)v_base, block_stride, block_size, n_kv_heads, head_dim, elem_bytes,
                       table, table_stride, unit_lens, chunk_rows, n_units, buf);
}

int oracle_kv_unpack_units(void* k_base, void* v_base, int64_t block_stride, int32_t block_size, int32_t n_kv_heads,
                           int32_t head_dim, int32_t elem_bytes, const int32_t* table, int32_t table_stride,
                           const int32_t* unit_lens, const int64_t* chunk_rows, int32_t n_units, const void* buf) {
  return kv_copy_units(0, k_base, v_base, block_stride, block_size, n_kv_heads, head_dim, elem_bytes, table,
                       table_stride, unit_lens, chunk_rows, n_units, (void*)buf);
}

/* Append: the new turn's K,V rows of one layer go into the paged cache behind the session's prefix, so that the next
 * turn (or decode step) finds them there (Sec. 2.1 "KV Cache": the keys and values of every processed token are kept;
 * Sec. 3.3: a finished request's new K,V blocks join the session's cache).  Token i of session s has position
 * P_s + i: block table[s][(P_s + i) / bs], slot (P_s + i) % bs.  Nothing else in the pools changes. */
int oracle_kv_append(void* k_base, void* v_base, int64_t layer_stride, int64_t block_stride, int32_t n_layers,
                     int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int32_t elem_bytes, int32_t layer,
                     const void* k_new, const void* v_new, const int32_t* cu_new_lens, const int32_t* prefix_lens,
                     const int32_t* table, int32_t table_stride, int32_t n_sessions) {
  if (elem_bytes != 2 && elem_bytes != 4) return -1;
  if (layer < 0 || layer >= n_layers) return -1;
  const int64_t row = (int64_t)n_kv_heads * head_dim;
  const size_t row_bytes = (size_t)row * elem_bytes;
  for (int32_t s = 0; s < n_sessions; ++s)
    for (int32_t i = 0; i < cu_new_lens[s + 1] - cu_new_lens[s]; ++i) {
      const int64_t pos = (int64_t)prefix_lens[s] + i;
      const int64_t b = table[(int64_t)s * table_stride + pos / block_size];
      const int64_t elem = (int64_t)layer * layer_stride + b * block_stride + (pos % block_size) * row;
      const int64_t src = ((int64_t)cu_new_lens[s] + i) * row;
      memcpy((char*)k_base + elem * elem_bytes, (const char*)k_new + src * elem_bytes, row_bytes);
      memcpy((char*)v_base + elem * elem_bytes, (const char*)v_new + src * elem_bytes, row_bytes);
    }
  return 0;
}

/* ------------------------------------------------------------------------------------------------------- */

static inline double widen(const void* base, int64_t idx, int is_bf16) {
  if (is_bf16) {
    uint32_t u = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
  }
  return (double)((const float*)base)[idx];
}

/* Key j (0 .. P+i) of session s for kv-head g: the pool (through the table) if j < P, else the new turn's row. */
static inline void key_location(int64_t j, int32_t P, int32_t g, const int32_t* table_row, int32_t block_size,
                                int64_t layer_off, int64_t block_stride, int32_t n_kv_heads, int32_t head_dim,
                                int32_t cu_s, int* in_pool, int64_t* elem) {
  if (j < P) {
    const int64_t b = table_row[j / block_size];
    const int64_t o = j % block_size;
    *in_pool = 1;
    *elem = layer_off + b * block_stride + (o * n_kv_heads + g) * head_dim;
  } else {
    *in_pool = 0;
    *elem = (((int64_t)cu_s + (j - P)) * n_kv_heads + g) * head_dim;
  }
}

/* Softmax weights and output of ONE query row (session s, new token i, query head h).
 * x_j = scale * <q, k_j>,  m = max_j x_j,  p_j = exp(x_j - m) / sum_j exp(x_j - m),  o = sum_j p_j v_j.
 * `weights` (P+i+1 doubles, may be NULL) receives p; `x` is caller scratch of the same length. */
static void attn_row(const void* k_base, const void* v_base, int64_t layer_off, int64_t block_stride,
                     int32_t block_size, int32_t n_kv_heads, int32_t head_dim, int is_bf16, const void* q,
                     const void* k_new, const void* v_new, int32_t n_q_heads, const int32_t* table_row, int32_t P,
                     int32_t cu_s, int32_t i, int32_t h, double scale, double* x, double* weights, double* o) {
  const int32_t G = n_q_heads / n_kv_heads;
  const int32_t g = h / G;
  const int64_t n_keys = (int64_t)P + i + 1;
  const int64_t q_off = (((int64_t)cu_s + i) * n_q_heads + h) * head_dim;
  double m = -INFINITY;
  for (int64_t j = 0; j < n_keys; ++j) {
    int in_pool;
    int64_t e;
    key_location(j, P, g, table_row, block_size, layer_off, block_stride, n_kv_heads, head_dim, cu_s, &in_pool, &e);
    const void* kb = in_pool ? k_base : k_new;
    double dot = 0.0;
    for (int32_t c = 0; c < head_dim; ++c) dot += widen(q, q_off + c, is_bf16) * widen(kb, e + c, is_bf16);
    x[j] = scale * dot;
    if (x[j] > m) m = x[j];
  }
  double Z = 0.0;
  for (int64_t j = 0; j < n_keys; ++j) {
    x[j] = exp(x[j] - m);
    Z += x[j];
  }
  for (int32_t c = 0; c < head_dim; ++c) o[c] = 0.0;
  for (int64_t j = 0; j < n_keys; ++j) {
    int in_pool;
    int64_t e;
    key_location(j, P, g, table_row, block_size, layer_off, block_stride, n_kv_heads, head_dim, cu_s, &in_pool, &e);
    const void* vb = in_pool ? v_base : v_new;
    const double p = x[j] / Z;
    if (weights) weights[j] = p;
    for (int32_t c = 0; c < head_dim; ++c) o[c] += p * widen(vb, e + c, is_bf16);
  }
}

/* Prefix-cached prefill attention of one layer, output in fp64: out[T][H_q][d].
 * token_subset: NULL to compute every new token, else n_subset global token indices (0 .. T-1) to compute,
 * all heads each; rows of other tokens are left untouched.  scale is the fp32 value the GPU path receives,
 * widened.  Returns 0, or -1 on a bad argument. */
int oracle_prefix_prefill_attn(const void* k_base, const void* v_base, int64_t layer_stride, int64_t block_stride,
                               int32_t layer, int32_t block_size, int32_t n_kv_heads, int32_t head_dim,
                               int32_t is_bf16, const void* q, const void* k_new, const void* v_new,
                               const int32_t* cu_new_lens, const int32_t* prefix_lens, const int32_t* table,
                               int32_t table_stride, int32_t n_sessions, int32_t n_q_heads, float scale,
                               const int32_t* token_subset, int32_t n_subset, double* out) {
  if (n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || head_dim <= 0 || block_size <= 0) return -1;
  const int64_t T = n_sessions > 0 ? cu_new_lens[n_sessions] : 0;
  const int64_t n_rows = token_subset ? n_subset : T;
  const int64_t layer_off = (int64_t)layer * layer_stride;
  int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
  for (int64_t r = 0; r < n_rows * n_q_heads; ++r) {
    const int64_t tok = token_subset ? token_subset[r / n_q_heads] : r / n_q_heads;
    const int32_t h = (int32_t)(r % n_q_heads);
    int32_t s = 0;
    while (s < n_sessions && cu_new_lens[s + 1] <= tok) ++s;
    if (s >= n_sessions || tok < 0) {
      bad |= 1;
      continue;
    }
    const int32_t i = (int32_t)(tok - cu_new_lens[s]);
    const int32_t P = prefix_lens[s];
    double* x = (double*)malloc(sizeof(double) * ((size_t)P + i + 1));
    attn_row(k_base, v_base, layer_off, block_stride, block_size, n_kv_heads, head_dim, is_bf16, q, k_new, v_new,
             n_q_heads, table + (int64_t)s * table_stride, P, cu_new_lens[s], i, h, (double)scale, x, NULL,
             out + (tok * n_q_heads + h) * head_dim);
    free(x);
  }
  return bad ? -1 : 0;
}

/* The softmax weights of one row (session s, new token i, head h): weights[0 .. P_s + i]. */
int oracle_attn_row_weights(const void* k_base, const void* v_base, int64_t layer_stride, int64_t block_stride,
                            int32_t layer, int32_t block_size, int32_t n_kv_heads, int32_t head_dim,
                            int32_t is_bf16, const void* q, const void* k_new, const void* v_new,
                            const int32_t* cu_new_lens, const int32_t* prefix_lens, const int32_t* table,
                            int32_t table_stride, int32_t n_q_heads, float scale, int32_t s, int32_t i, int32_t h,
                            double* weights, double* o) {
  const int32_t P = prefix_lens[s];
  double* x = (double*)malloc(sizeof(double) * ((size_t)P + i + 1));
  attn_row(k_base, v_base, (int64_t)layer * layer_stride, block_stride, block_size, n_kv_heads, head_dim, is_bf16,
           q, k_new, v_new, n_q_heads, table + (int64_t)s * table_stride, P, cu_new_lens[s], i, h, (double)scale,
           x, weights, o);
  free(x);
  return 0;
}
