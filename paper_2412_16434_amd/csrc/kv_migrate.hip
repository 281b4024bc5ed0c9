// kv_pack / kv_unpack: gather a session's scattered K,V blocks into the layer-major migration buffer and
// scatter an arrived buffer into free-list blocks (Symphony Sec. 3.2 node manager, Sec. 3.3 memory management).
//
// The operation is a permutation copy, bound by HBM bandwidth.  Work decomposition:
//   * the unit of indirection is one token row (n_kv_heads*head_dim elements, 2 KiB for Llama-3.1 shapes), which
//     is contiguous both in the pool and in the buffer, so partially filled last blocks need no special path;
//   * one lane owns one 16-byte vector of one token row and moves that vector for PLANES consecutive
//     (layer, K|V) planes: the session lookup and the block-table read are done once and reused for every
//     plane, and all PLANES loads are issued before the first store so each wave keeps PLANES KiB in flight;
//   * blockIdx.x walks the global token space (adjacent workgroups touch adjacent rows of the same plane),
//     blockIdx.y walks groups of planes.
#include "common.h"

#include <stdlib.h>

namespace symph {

struct MigrateParams {
  char* k_base;
  char* v_base;
  int64_t layer_stride_b;  // bytes
  int64_t block_stride_b;  // bytes
  int32_t row_bytes;
  int32_t vecs_per_row;
  int32_t block_size;
  int32_t n_blocks;
  int32_t n_planes;  // 2 * n_layers
  const int32_t* table;
  int32_t table_stride;
  const int32_t* prefix_lens;
  const int64_t* offsets;
  int32_t n_sessions;
  int64_t total_tokens;
  char* buf;
  int64_t buf_bytes;
};

template <typename VecT, bool NT>
__device__ __forceinline__ VecT load_vec(const char* p) {
  if constexpr (NT)
    return __builtin_nontemporal_load(reinterpret_cast<const VecT*>(p));
  else
    return *reinterpret_cast<const VecT*>(p);
}

template <typename VecT, bool NT>
__device__ __forceinline__ void store_vec(char* p, VecT v) {
  if constexpr (NT)
    __builtin_nontemporal_store(v, reinterpret_cast<VecT*>(p));
  else
    *reinterpret_cast<VecT*>(p) = v;
}

template <typename VecT, bool PACK, int PLANES, bool NT>
__global__ __launch_bounds__(256) void kv_migrate_kernel(const MigrateParams p) {
  const int64_t gv = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t tg = gv / p.vecs_per_row;  // token in the concatenated token space of all sessions
  if (tg >= p.total_tokens) return;
  const int32_t col = (int32_t)(gv - tg * p.vecs_per_row);

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
  const int32_t P = p.prefix_lens[s];
  const int64_t t = tg - off_s;
  if (t >= P) return;  // inconsistent offsets / lengths: touch nothing
  const int32_t j = (int32_t)(t / p.block_size);
  if (j >= p.table_stride) return;
  const int32_t b = p.table[(int64_t)s * p.table_stride + j];
  if (b < 0 || b >= p.n_blocks) return;  // not a block of this cache: touch nothing
  const int32_t slot = (int32_t)(t - (int64_t)j * p.block_size);

  const int64_t pool_off = (int64_t)b * p.block_stride_b + (int64_t)slot * p.row_bytes + (int64_t)col * sizeof(VecT);
  const int64_t plane_b = (int64_t)P * p.row_bytes;  // one (layer, K|V) plane of this session in the buffer
  const int64_t buf_off0 = off_s * p.n_planes * p.row_bytes + t * p.row_bytes + (int64_t)col * sizeof(VecT);

  const int32_t plane0 = blockIdx.y * PLANES;
  VecT v[PLANES];
#pragma unroll
  for (int i = 0; i < PLANES; ++i) {
    const int32_t pl = plane0 + i;
    if (pl < p.n_planes) {
      const int64_t bo = buf_off0 + pl * plane_b;
      const char* pool = ((pl & 1) ? p.v_base : p.k_base) + (int64_t)(pl >> 1) * p.layer_stride_b + pool_off;
      if (bo + (int64_t)sizeof(VecT) <= p.buf_bytes) v[i] = PACK ? load_vec<VecT, NT>(pool) : load_vec<VecT, NT>(p.buf + bo);
    }
  }
#pragma unroll
  for (int i = 0; i < PLANES; ++i) {
    const int32_t pl = plane0 + i;
    if (pl < p.n_planes) {
      const int64_t bo = buf_off0 + pl * plane_b;
      char* pool = ((pl & 1) ? p.v_base : p.k_base) + (int64_t)(pl >> 1) * p.layer_stride_b + pool_off;
      if (bo + (int64_t)sizeof(VecT) <= p.buf_bytes) {
        if (PACK)
          store_vec<VecT, NT>(p.buf + bo, v[i]);
        else
          store_vec<VecT, NT>(pool, v[i]);
      }
    }
  }
}

template <typename VecT, bool PACK, int PLANES>
static void launch_nt(bool nt, dim3 grid, const MigrateParams& p, hipStream_t stream) {
  if (nt)
    hipLaunchKernelGGL((kv_migrate_kernel<VecT, PACK, PLANES, true>), grid, dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL((kv_migrate_kernel<VecT, PACK, PLANES, false>), grid, dim3(256), 0, stream, p);
}

template <typename VecT, bool PACK>
static int32_t launch_planes(int planes, bool nt, const MigrateParams& p, hipStream_t stream) {
  const int64_t n_vec = p.total_tokens * p.vecs_per_row;
  const int64_t gx = ceil_div64(n_vec, 256);
  const int64_t gy = ceil_div64(p.n_planes, planes);
  if (gx > 0x7FFFFFFFLL || gy > 65535) return SYMPH_EUNSUPPORTED;
  dim3 grid((unsigned)gx, (unsigned)gy);
  switch (planes) {
    case 2: launch_nt<VecT, PACK, 2>(nt, grid, p, stream); break;
    case 4: launch_nt<VecT, PACK, 4>(nt, grid, p, stream); break;
    case 8: launch_nt<VecT, PACK, 8>(nt, grid, p, stream); break;
    default: return SYMPH_EINVAL;
  }
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

static int env_int(const char* name, int dflt) {
  const char* e = getenv(name);
  return e ? atoi(e) : dflt;
}

int32_t launch_kv_migrate(bool pack, const symph_kv_cache* c, const int32_t* d_table, int32_t table_stride,
                          const int32_t* d_prefix_lens, const int64_t* d_offsets, int32_t n_sessions,
                          int64_t total_tokens, void* d_buf, int64_t buf_bytes, hipStream_t stream) {
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
  p.block_size = c->block_size;
  p.n_blocks = c->n_blocks;
  p.n_planes = 2 * c->n_layers;
  p.table = d_table;
  p.table_stride = table_stride;
  p.prefix_lens = d_prefix_lens;
  p.offsets = d_offsets;
  p.n_sessions = n_sessions;
  p.total_tokens = total_tokens;
  p.buf = (char*)d_buf;
  p.buf_bytes = buf_bytes;

  // Tuning knobs (development): planes per lane and non-temporal access.
  int planes = env_int("SYMPH_MIGRATE_PLANES", 8);
  if (planes != 2 && planes != 4 && planes != 8) planes = 8;
  while (planes > 2 && planes > p.n_planes) planes >>= 1;
  const bool nt = env_int("SYMPH_MIGRATE_NT", 1) != 0;

  if (vec == 16) return pack ? launch_planes<u32x4, true>(planes, nt, p, stream) : launch_planes<u32x4, false>(planes, nt, p, stream);
  return pack ? launch_planes<unsigned int, true>(planes, nt, p, stream)
              : launch_planes<unsigned int, false>(planes, nt, p, stream);
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
  constexpr int UNROLL = 8;
  const int64_t n_vec = bytes / 16;
  const int64_t g = ceil_div64(n_vec, 256 * UNROLL);
  if (g > 0x7FFFFFFFLL) return SYMPH_EUNSUPPORTED;
  hipLaunchKernelGGL((device_copy_kernel<UNROLL>), dim3((unsigned)g), dim3(256), 0, stream, (u32x4*)d_dst,
                     (const u32x4*)d_src, n_vec);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

}  // namespace symph
