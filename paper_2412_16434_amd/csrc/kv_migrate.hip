// kv_pack / kv_unpack: gather a session's scattered K,V blocks into the layer-major migration buffer and
// scatter an arrived buffer into free-list blocks (Symphony Sec. 3.2 node manager, Sec. 3.3 memory management).
//
// The operation is a permutation copy, bound by HBM bandwidth.  Work decomposition:
//   * the unit of indirection is one token row (n_kv_heads*head_dim elements, 2 KiB for Llama-3.1 shapes), which
//     is contiguous both in the pool and in the buffer, so partially filled last blocks need no special path;
//   * one lane owns one 16-byte vector of one token row and moves that vector for PLANES (1 or 2) consecutive
//     (layer, K|V) planes; the session lookup and the block-table read are wave-uniform and run on the scalar
//     unit; loads are issued before the stores.  Little is kept in flight per lane on purpose: on MI355X one
//     vector per lane and a very wide grid copies fastest (eight per lane loses a third of the bandwidth);
//   * blockIdx.x walks the global token space (adjacent workgroups touch adjacent rows of the same plane),
//     blockIdx.y walks groups of planes.
#include "common.h"

namespace symph {

struct MigrateParams {
  char* k_base;
  char* v_base;
  int64_t layer_stride_b;  // bytes
  int64_t block_stride_b;  // bytes
  int32_t row_bytes;
  int32_t vecs_per_row;
  int32_t row_shift;  // log2(vecs_per_row) when it is a power of two, else -1
  int32_t block_size;
  int32_t bs_shift;   // log2(block_size) when it is a power of two, else -1
  int32_t n_blocks;
  int32_t n_planes;  // 2 * n_layers
  int32_t plane_begin, plane_end;  // planes moved by this launch (a range of layers: 2 * layer_begin .. 2 * layer_end)
  const int32_t* table;
  int32_t table_stride;
  const int32_t* prefix_lens;
  const int32_t* tail_begin;  // null: whole sessions; else only tokens tail_begin[s] .. prefix_lens[s]-1 move, and
                              // offsets / total_tokens count those
  const int64_t* offsets;
  const int64_t* chunk_rows;  // null: session s starts at row offsets[s] * n_planes of the buffer (whole-cache layout);
                              // else at row chunk_rows[s] (units of one layer placed anywhere in a larger buffer)
  int32_t n_sessions;
  int64_t total_tokens;
  char* buf;
  int64_t buf_bytes;
  int32_t xcd_chunk;  // > 0: workgroups per XCD in the XCD-contiguous mapping of blockIdx.x; 0: identity mapping
  int64_t batch_layer_b;  // 0: session-major buffer (a session's layers follow each other); else the bytes of one layer
                          // of the WHOLE batch in the layer-major buffer (layer, then session, then K|V, then token)
};

template <typename VecT, int NT>
__device__ __forceinline__ VecT load_vec(const char* p) {
  if constexpr (NT & 1)
    return __builtin_nontemporal_load(reinterpret_cast<const VecT*>(p));
  else
    return *reinterpret_cast<const VecT*>(p);
}

template <typename VecT, int NT>
__device__ __forceinline__ void store_vec(char* p, VecT v) {
  if constexpr (NT & 2)
    __builtin_nontemporal_store(v, reinterpret_cast<VecT*>(p));
  else
    *reinterpret_cast<VecT*>(p) = v;
}

// UNIFORM: a token row is a whole number of waves (vecs_per_row is a power of two >= 64), so the token index, the
// session search and the block-table read are wave-uniform and run once per wave on the scalar unit.
template <typename VecT, bool PACK, int PLANES, int NT, bool UNIFORM>
__global__ __launch_bounds__(256) void kv_migrate_kernel(const MigrateParams p) {
  // Workgroups are dealt round-robin to the 8 XCDs.  With the XCD-contiguous mapping, XCD x walks the x-th eighth of
  // the token space, so the rows of one pool block (consecutive workgroups in the mapped order) are moved by one XCD.
  int64_t wg = blockIdx.x;
  if (p.xcd_chunk > 0 && wg < 8 * (int64_t)p.xcd_chunk) wg = (wg & 7) * (int64_t)p.xcd_chunk + (wg >> 3);
  const int64_t gv = wg * 256 + threadIdx.x;
  int64_t tg;  // token in the concatenated token space of all sessions
  int32_t col;
  if constexpr (UNIFORM) {
    const int64_t t64 = gv >> p.row_shift;
    col = (int32_t)gv & (p.vecs_per_row - 1);
    tg = ((int64_t)__builtin_amdgcn_readfirstlane((int32_t)(t64 >> 32)) << 32) |
         (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)t64);
  } else {
    tg = p.row_shift >= 0 ? (gv >> p.row_shift) : gv / p.vecs_per_row;
    col = (int32_t)(gv - tg * p.vecs_per_row);
  }
  if (tg >= p.total_tokens) return;

  // session s with offsets[s] <= tg < offsets[s+1] (sessions of length 0 are skipped by taking the last match)
  int32_t lo = 0, hi = p.n_sessions;
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (p.offsets[mid] <= tg)
      lo = mid;
    else
      hi = mid;
  }
  const int32_t s = lo;
  const int64_t off_s = p.offsets[s];
  const int32_t first = p.tail_begin ? p.tail_begin[s] : 0;
  const int32_t P = p.prefix_lens[s] - first;  // tokens of this session in the buffer
  const int64_t t64 = tg - off_s;
  if (first < 0 || t64 >= P) return;  // inconsistent offsets / lengths: touch nothing
  const int32_t t = first + (int32_t)t64;  // position in the session
  const int32_t j = p.bs_shift >= 0 ? (t >> p.bs_shift) : t / p.block_size;
  if (j >= p.table_stride) return;
  const int32_t b = p.table[(int64_t)s * p.table_stride + j];
  if (b < 0 || b >= p.n_blocks) return;  // not a block of this cache: touch nothing
  const int32_t slot = t - j * p.block_size;
  // Plane pl = (layer, K|V) of this session starts at sess_b + (pl / 2) * layer_b + (pl % 2) * plane_b of the buffer.
  const int64_t plane_b = (int64_t)P * p.row_bytes;
  int64_t sess_b = off_s * p.n_planes * p.row_bytes;
  int64_t layer_b = 2 * plane_b;
  if (p.batch_layer_b) {
    sess_b = off_s * 2 * p.row_bytes;
    layer_b = p.batch_layer_b;
  }
  if (p.chunk_rows) {
    const int64_t first_row = p.chunk_rows[s];
    if (first_row < 0 || first_row > p.buf_bytes / p.row_bytes) return;  // (the second test also keeps the product in range)
    sess_b = first_row * p.row_bytes;
  }
  // the session's last plane would not fit the buffer: touch nothing
  if (sess_b + (int64_t)(p.n_planes / 2 - 1) * layer_b + 2 * plane_b > p.buf_bytes) return;

  const int64_t pool_off = (int64_t)b * p.block_stride_b + (int64_t)slot * p.row_bytes + (int64_t)col * sizeof(VecT);
  const int64_t buf_off0 = sess_b + t64 * p.row_bytes + (int64_t)col * sizeof(VecT);

  const int32_t plane0 = p.plane_begin + blockIdx.y * PLANES;
  VecT v[PLANES];
#pragma unroll
  for (int i = 0; i < PLANES; ++i) {
    const int32_t pl = min(plane0 + i, p.plane_end - 1);  // a ragged last group repeats its last plane (same bytes)
    const char* pool = ((pl & 1) ? p.v_base : p.k_base) + (int64_t)(pl >> 1) * p.layer_stride_b + pool_off;
    v[i] = PACK ? load_vec<VecT, NT>(pool) : load_vec<VecT, NT>(p.buf + buf_off0 + (pl >> 1) * layer_b + (pl & 1) * plane_b);
  }
#pragma unroll
  for (int i = 0; i < PLANES; ++i) {
    const int32_t pl = min(plane0 + i, p.plane_end - 1);
    char* pool = ((pl & 1) ? p.v_base : p.k_base) + (int64_t)(pl >> 1) * p.layer_stride_b + pool_off;
    if (PACK)
      store_vec<VecT, NT>(p.buf + buf_off0 + (pl >> 1) * layer_b + (pl & 1) * plane_b, v[i]);
    else
      store_vec<VecT, NT>(pool, v[i]);
  }
}

// The same copy with ROWS consecutive tokens per wave (rows that fill whole waves only).  A wave's life is a chain of
// dependent scalar loads (session search, lengths, block id) followed by one vector load and one store; with every
// wave slot of the chip taken, the bytes in flight are the waves in their load phase, so a wave that pays for the
// chain once and then has ROWS loads in flight keeps more of the memory system busy.  The session of the first token
// is searched for; the following tokens step to the next session when they pass its end.
template <typename VecT, bool PACK, int ROWS, int PLANES, int NT>
__global__ __launch_bounds__(256) void kv_migrate_rows_kernel(const MigrateParams p) {
  int64_t wg = blockIdx.x;
  if (p.xcd_chunk > 0 && wg < 8 * (int64_t)p.xcd_chunk) wg = (wg & 7) * (int64_t)p.xcd_chunk + (wg >> 3);
  const int lane = threadIdx.x & 63;
  const int64_t wave64 = wg * 4 + (threadIdx.x >> 6);
  const int64_t wave_id = ((int64_t)__builtin_amdgcn_readfirstlane((int32_t)(wave64 >> 32)) << 32) |
                          (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)wave64);
  const int wave_shift = p.row_shift - 6;                       // log2(waves per row)
  const int64_t tg0 = (wave_id >> wave_shift) * ROWS;           // first token of this wave, in the concatenated space
  const int32_t col = ((int32_t)(wave_id & ((1 << wave_shift) - 1)) << 6) + lane;
  if (tg0 >= p.total_tokens) return;

  int32_t lo = 0, hi = p.n_sessions;   // session s with offsets[s] <= tg0 < offsets[s+1] (the last match skips empty ones)
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (p.offsets[mid] <= tg0)
      lo = mid;
    else
      hi = mid;
  }
  int32_t s = lo;
  int64_t off_s = p.offsets[s], off_next = p.offsets[s + 1];
  int64_t pool_off[ROWS], buf_off[ROWS], layer_b[ROWS], plane_b[ROWS];
  bool ok[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    const int64_t tg = tg0 + r;
    ok[r] = tg < p.total_tokens;
    if (ok[r])
      while (tg >= off_next && s + 1 < p.n_sessions) {   // past the end of the session: the next one with tokens
        ++s;
        off_s = off_next;
        off_next = p.offsets[s + 1];
      }
    const int32_t first = p.tail_begin ? p.tail_begin[s] : 0;
    const int32_t P = p.prefix_lens[s] - first;
    const int64_t t64 = tg - off_s;
    ok[r] = ok[r] && first >= 0 && t64 >= 0 && t64 < P;   // inconsistent offsets / lengths: touch nothing
    const int32_t t = first + (int32_t)t64;
    const int32_t j = p.bs_shift >= 0 ? (t >> p.bs_shift) : t / p.block_size;
    ok[r] = ok[r] && j >= 0 && j < p.table_stride;
    const int32_t b = ok[r] ? p.table[(int64_t)s * p.table_stride + j] : -1;
    ok[r] = ok[r] && b >= 0 && b < p.n_blocks;            // not a block of this cache: touch nothing
    const int32_t slot = t - j * p.block_size;
    plane_b[r] = (int64_t)P * p.row_bytes;
    layer_b[r] = 2 * plane_b[r];
    int64_t sess_b = off_s * p.n_planes * p.row_bytes;
    if (p.batch_layer_b) {
      sess_b = off_s * 2 * p.row_bytes;
      layer_b[r] = p.batch_layer_b;
    }
    if (p.chunk_rows) {
      const int64_t first_row = ok[r] ? p.chunk_rows[s] : 0;
      ok[r] = ok[r] && first_row >= 0 && first_row <= p.buf_bytes / p.row_bytes;
      sess_b = first_row * p.row_bytes;
    }
    ok[r] = ok[r] && sess_b + (int64_t)(p.n_planes / 2 - 1) * layer_b[r] + 2 * plane_b[r] <= p.buf_bytes;
    pool_off[r] = (int64_t)b * p.block_stride_b + (int64_t)slot * p.row_bytes + (int64_t)col * sizeof(VecT);
    buf_off[r] = sess_b + t64 * p.row_bytes + (int64_t)col * sizeof(VecT);
  }

  const int32_t plane0 = p.plane_begin + blockIdx.y * PLANES;
  VecT v[ROWS][PLANES];
#pragma unroll
  for (int r = 0; r < ROWS; ++r)
#pragma unroll
    for (int i = 0; i < PLANES; ++i) {
      const int32_t pl = min(plane0 + i, p.plane_end - 1);  // a ragged last group repeats its last plane (same bytes)
      const char* pool = ((pl & 1) ? p.v_base : p.k_base) + (int64_t)(pl >> 1) * p.layer_stride_b + pool_off[r];
      const char* in_buf = p.buf + buf_off[r] + (pl >> 1) * layer_b[r] + (pl & 1) * plane_b[r];
      if (ok[r]) v[r][i] = load_vec<VecT, NT>(PACK ? pool : in_buf);
    }
#pragma unroll
  for (int r = 0; r < ROWS; ++r)
#pragma unroll
    for (int i = 0; i < PLANES; ++i) {
      const int32_t pl = min(plane0 + i, p.plane_end - 1);
      char* pool = ((pl & 1) ? p.v_base : p.k_base) + (int64_t)(pl >> 1) * p.layer_stride_b + pool_off[r];
      char* in_buf = p.buf + buf_off[r] + (pl >> 1) * layer_b[r] + (pl & 1) * plane_b[r];
      if (ok[r]) store_vec<VecT, NT>(PACK ? in_buf : pool, v[r][i]);
    }
}

// Non-temporal loads and stores (every byte is touched once): bit 0 loads, bit 1 stores.
constexpr int kMigrateNT = 3;

template <typename VecT, bool PACK, int PLANES>
static void launch_uniform(dim3 grid, const MigrateParams& p, hipStream_t stream) {
  if (p.row_shift >= 6)  // a row is a whole number of waves: scalar session search and table read
    hipLaunchKernelGGL((kv_migrate_kernel<VecT, PACK, PLANES, kMigrateNT, true>), grid, dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL((kv_migrate_kernel<VecT, PACK, PLANES, kMigrateNT, false>), grid, dim3(256), 0, stream, p);
}

template <typename VecT, bool PACK, int ROWS, int PLANES>
static int32_t launch_rows(const MigrateParams& p_in, hipStream_t stream) {
  const int64_t n_vec = ceil_div64(p_in.total_tokens, ROWS) * p_in.vecs_per_row;
  const int64_t gx = ceil_div64(n_vec, 256);
  const int64_t gy = ceil_div64(p_in.plane_end - p_in.plane_begin, PLANES);
  if (gx > 0x7FFFFFFFLL || gy > 65535) return SYMPH_EUNSUPPORTED;
  MigrateParams p = p_in;
  p.xcd_chunk = PACK ? (int32_t)(gx / 8) : 0;
  hipLaunchKernelGGL((kv_migrate_rows_kernel<VecT, PACK, ROWS, PLANES, kMigrateNT>), dim3((unsigned)gx, (unsigned)gy),
                     dim3(256), 0, stream, p);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

template <typename VecT, bool PACK>
static int32_t launch_planes(int planes, const MigrateParams& p_in, hipStream_t stream) {
  // Measured on MI355X, gather with one plane per lane: two consecutive tokens per wave, i.e. one session search for
  // two loads, +5 % on config 2 (16 sessions: 5.8 -> 6.1 TB/s), four the same, eight a cliff (3.1 TB/s); nothing to
  // gain with a single session (no search: 6.08 -> 5.99) or in the two-plane form (config 4: 6.5 either way), and the
  // scatter does not change (6.5 / 5.3 / 5.2 TB/s on configs 2 / 4 / 3 with one, two or four tokens per wave).
  if (PACK && planes == 1 && p_in.row_shift >= 6 && p_in.n_sessions > 1) return launch_rows<VecT, PACK, 2, 1>(p_in, stream);
  const int64_t n_vec = p_in.total_tokens * p_in.vecs_per_row;
  const int64_t gx = ceil_div64(n_vec, 256);
  const int64_t gy = ceil_div64(p_in.plane_end - p_in.plane_begin, planes);
  if (gx > 0x7FFFFFFFLL || gy > 65535) return SYMPH_EUNSUPPORTED;
  dim3 grid((unsigned)gx, (unsigned)gy);
  MigrateParams p = p_in;
  // measured on MI355X (config 2): the gather gains 2-3 % from the XCD-contiguous mapping, the scatter loses 7 %
  p.xcd_chunk = PACK ? (int32_t)(gx / 8) : 0;
  if (planes == 1)
    launch_uniform<VecT, PACK, 1>(grid, p, stream);
  else
    launch_uniform<VecT, PACK, 2>(grid, p, stream);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

static int log2_or_neg(int64_t x) { return (x > 0 && (x & (x - 1)) == 0) ? __builtin_ctzll((unsigned long long)x) : -1; }

int32_t launch_kv_migrate(bool pack, const symph_kv_cache* c, int32_t layer_begin, int32_t layer_end,
                          const int32_t* d_table, int32_t table_stride, const int32_t* d_prefix_lens,
                          const int32_t* d_tail_begin, const int64_t* d_offsets, int32_t n_sessions,
                          int64_t total_tokens, void* d_buf, int64_t buf_bytes, hipStream_t stream,
                          const int64_t* d_chunk_rows, bool batch_layer_major) {
  const int eb = elem_bytes_of(c->dtype);
  const int64_t row_bytes = (int64_t)c->n_kv_heads * c->head_dim * eb;
  if (row_bytes > 0x7FFFFFFF) return SYMPH_EUNSUPPORTED;
  // widest vector that divides the row and every base / stride
  const uintptr_t align_or = (uintptr_t)c->k_base | (uintptr_t)c->v_base | (uintptr_t)d_buf |
                             (uintptr_t)(c->layer_stride * eb) | (uintptr_t)(c->block_stride * eb) |
                             (uintptr_t)row_bytes;
  int vec = 16;
  if (align_or & 15) vec = 4;
  if (align_or & 3) return SYMPH_EUNSUPPORTED;

  MigrateParams p;
  p.k_base = (char*)c->k_base;
  p.v_base = (char*)c->v_base;
  p.layer_stride_b = c->layer_stride * eb;
  p.block_stride_b = c->block_stride * eb;
  p.row_bytes = (int32_t)row_bytes;
  p.vecs_per_row = (int32_t)(row_bytes / vec);
  p.row_shift = log2_or_neg(p.vecs_per_row);
  p.block_size = c->block_size;
  p.bs_shift = log2_or_neg(c->block_size);
  p.n_blocks = c->n_blocks;
  p.n_planes = 2 * c->n_layers;
  p.plane_begin = 2 * layer_begin;
  p.plane_end = 2 * layer_end;
  p.table = d_table;
  p.table_stride = table_stride;
  p.prefix_lens = d_prefix_lens;
  p.tail_begin = d_tail_begin;
  p.offsets = d_offsets;
  p.chunk_rows = d_chunk_rows;
  p.n_sessions = n_sessions;
  p.total_tokens = total_tokens;
  p.buf = (char*)d_buf;
  p.buf_bytes = buf_bytes;
  p.batch_layer_b = batch_layer_major ? 2 * total_tokens * row_bytes : 0;

  // Planes per lane, measured on MI355X (config 2 / config 4, TB/s read+written): gather 1 -> 6.1 / 5.6,
  // 2 -> 5.8 / 5.9, 4 -> 5.5 / 5.7, 8 -> 3.0; scatter 1 -> 5.9 / 5.5, 2 -> 6.5 / 6.2, 4 -> 6.3 / 6.2.  One plane per
  // lane repeats the session search for every vector, which only pays off while the search is short.
  const int planes = (pack && n_sessions <= 64) ? 1 : 2;  // (a launch always covers whole layers: two planes at least)

  if (vec == 16) return pack ? launch_planes<u32x4, true>(planes, p, stream) : launch_planes<u32x4, false>(planes, p, stream);
  return pack ? launch_planes<unsigned int, true>(planes, p, stream) : launch_planes<unsigned int, false>(planes, p, stream);
}

// ------------------------------------------------------------------------------------------------------------
// append of the new turn's rows (one layer)
// ------------------------------------------------------------------------------------------------------------
struct AppendParams {
  char* k_layer;  // the layer's K pool and V pool
  char* v_layer;
  int64_t block_stride_b;
  int32_t row_bytes, vecs_per_row, block_size, n_blocks;
  const char* k_new;
  const char* v_new;
  const int32_t* cu_new_lens;
  const int32_t* prefix_lens;
  const int32_t* table;
  int32_t table_stride, n_sessions, total_new_tokens;
};

// One lane moves one vector of one new token's row, for K and for V.
template <typename VecT>
__global__ __launch_bounds__(256) void kv_append_kernel(const AppendParams p) {
  const int64_t gv = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t tok = gv / p.vecs_per_row;
  if (tok >= p.total_new_tokens) return;
  const int32_t col = (int32_t)(gv - tok * p.vecs_per_row);
  int32_t lo = 0, hi = p.n_sessions;  // last session with cu[s] <= tok (empty turns are skipped this way)
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (p.cu_new_lens[mid] <= tok)
      lo = mid;
    else
      hi = mid;
  }
  const int32_t s = lo;
  const int64_t pos = (int64_t)p.prefix_lens[s] + (tok - p.cu_new_lens[s]);
  if (pos < 0) return;
  const int64_t j = pos / p.block_size;
  if (j >= p.table_stride) return;
  const int32_t b = p.table[(int64_t)s * p.table_stride + j];
  if (b < 0 || b >= p.n_blocks) return;  // not a block of this cache: touch nothing
  const int64_t dst = (int64_t)b * p.block_stride_b + (pos - j * p.block_size) * p.row_bytes + (int64_t)col * sizeof(VecT);
  const int64_t src = tok * p.row_bytes + (int64_t)col * sizeof(VecT);
  const VecT kv = *reinterpret_cast<const VecT*>(p.k_new + src);
  const VecT vv = *reinterpret_cast<const VecT*>(p.v_new + src);
  *reinterpret_cast<VecT*>(p.k_layer + dst) = kv;
  *reinterpret_cast<VecT*>(p.v_layer + dst) = vv;
}

int32_t launch_kv_append(const symph_kv_cache* c, int32_t layer, const void* d_k_new, const void* d_v_new,
                         const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens, const int32_t* d_table,
                         int32_t table_stride, int32_t n_sessions, int32_t total_new_tokens, hipStream_t stream) {
  const int eb = elem_bytes_of(c->dtype);
  const int64_t row_bytes = (int64_t)c->n_kv_heads * c->head_dim * eb;
  if (row_bytes > 0x7FFFFFFF) return SYMPH_EUNSUPPORTED;
  AppendParams p;
  p.k_layer = (char*)c->k_base + (int64_t)layer * c->layer_stride * eb;
  p.v_layer = (char*)c->v_base + (int64_t)layer * c->layer_stride * eb;
  p.block_stride_b = c->block_stride * eb;
  const uintptr_t align_or = (uintptr_t)p.k_layer | (uintptr_t)p.v_layer | (uintptr_t)d_k_new | (uintptr_t)d_v_new |
                             (uintptr_t)p.block_stride_b | (uintptr_t)row_bytes;
  if (align_or & 3) return SYMPH_EUNSUPPORTED;
  const int vec = (align_or & 15) ? 4 : 16;
  p.row_bytes = (int32_t)row_bytes;
  p.vecs_per_row = (int32_t)(row_bytes / vec);
  p.block_size = c->block_size;
  p.n_blocks = c->n_blocks;
  p.k_new = (const char*)d_k_new;
  p.v_new = (const char*)d_v_new;
  p.cu_new_lens = d_cu_new_lens;
  p.prefix_lens = d_prefix_lens;
  p.table = d_table;
  p.table_stride = table_stride;
  p.n_sessions = n_sessions;
  p.total_new_tokens = total_new_tokens;
  const int64_t g = ceil_div64((int64_t)total_new_tokens * p.vecs_per_row, 256);
  if (g > 0x7FFFFFFFLL) return SYMPH_EUNSUPPORTED;
  if (vec == 16)
    hipLaunchKernelGGL(kv_append_kernel<u32x4>, dim3((unsigned)g), dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL(kv_append_kernel<unsigned int>, dim3((unsigned)g), dim3(256), 0, stream, p);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

// ------------------------------------------------------------------------------------------------------------
// contiguous reference copy
// ------------------------------------------------------------------------------------------------------------
template <int UNROLL>
__global__ __launch_bounds__(256) void device_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                          int64_t n_vec) {
  const int64_t base = ((int64_t)blockIdx.x * UNROLL) * 256 + threadIdx.x;
  u32x4 v[UNROLL];
#pragma unroll
  for (int i = 0; i < UNROLL; ++i) {
    const int64_t k = base + (int64_t)i * 256;
    if (k < n_vec) v[i] = __builtin_nontemporal_load(src + k);
  }
#pragma unroll
  for (int i = 0; i < UNROLL; ++i) {
    const int64_t k = base + (int64_t)i * 256;
    if (k < n_vec) __builtin_nontemporal_store(v[i], dst + k);
  }
}

int32_t launch_device_copy(void* d_dst, const void* d_src, int64_t bytes, hipStream_t stream) {
  constexpr int UNROLL = 1;  // one 16-byte vector per lane and a very wide grid measured fastest on MI355X
  const int64_t n_vec = bytes / 16;
  const int64_t g = ceil_div64(n_vec, 256 * UNROLL);
  if (g > 0x7FFFFFFFLL) return SYMPH_EUNSUPPORTED;
  hipLaunchKernelGGL((device_copy_kernel<UNROLL>), dim3((unsigned)g), dim3(256), 0, stream, (u32x4*)d_dst,
                     (const u32x4*)d_src, n_vec);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

}  // namespace symph
