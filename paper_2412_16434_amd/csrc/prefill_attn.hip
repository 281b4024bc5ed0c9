// prefix_prefill_attn: the new turn's GQA queries against [paged cached prefix ; causal new tokens]
// (Symphony Sec. 2.1: A_h = softmax(Q_h K_h^T * scale), y = concat_h A_h V_h; a token sees all prior tokens).
//
// bf16 path (head_dim 128), one workgroup of 4 waves per (session, kv-head, tile of query tokens):
//   * the G query heads that share a kv-head are stacked into the tile (128 query rows = G heads x 128/G tokens),
//     so every K,V tile staged in LDS is reused by all of them;
//   * scores are computed TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: the MFMA result layout then puts
//     one query per lane, so the online-softmax statistics (running max, running sum, rescale factor) are per-lane
//     scalars, and the bf16 probabilities a lane holds are exactly the B operand of O^T += V^T P^T;
//   * the row order in which K rows are fed to the MFMA is permuted so that the 8 probabilities a lane needs for
//     one 16-key step of the second product are 8 consecutive keys, read from V^T in LDS with one 16-byte load;
//   * K,V tiles of 64 keys are fetched from the paged pool (block-table indirection per 16-token block) or from
//     the contiguous new-turn K,V, prefetched into registers while the previous tile is being multiplied.
// generic path (fp32, or head_dim 64): one wave per query row, lanes over keys, fp32 online softmax.
#include "common.h"

#include <stdlib.h>

#include <type_traits>

// Development-only timing ablations (never defined in the product build): bit 0 skips the softmax arithmetic,
// bit 1 the global loads and staging after the prologue, bit 2 the P*V product, bit 3 the Q*K product.
#ifndef SYMPH_DEV_ABLATE
#define SYMPH_DEV_ABLATE 0
#endif

namespace symph {

// ------------------------------------------------------------------------------------------------------------
// generic path: one wave per (token, query head)
// ------------------------------------------------------------------------------------------------------------
struct GenericParams {
  const void* k_layer;
  const void* v_layer;
  int64_t block_stride;
  int32_t n_blocks, block_size, n_kv_heads, n_q_heads;
  const void* q;
  const void* k_new;
  const void* v_new;
  void* out;
  const int32_t* cu_new_lens;
  const int32_t* prefix_lens;
  const int32_t* table;
  int32_t table_stride, n_sessions, total_new_tokens;
  float scale;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__bf16 x) { return (float)x; }
__device__ __forceinline__ void from_f32(float* p, float x) { *p = x; }
__device__ __forceinline__ void from_f32(__bf16* p, float x) { *p = (__bf16)x; }

template <typename T, int D>
__global__ __launch_bounds__(64) void attn_generic_kernel(const GenericParams p) {
  __shared__ float q_s[D];
  const int64_t row = blockIdx.x;  // (token, head)
  const int32_t tok = (int32_t)(row / p.n_q_heads);
  const int32_t h = (int32_t)(row % p.n_q_heads);
  const int lane = threadIdx.x;

  int32_t lo = 0, hi = p.n_sessions;  // session with cu[s] <= tok < cu[s+1]
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (p.cu_new_lens[mid] <= tok)
      lo = mid;
    else
      hi = mid;
  }
  const int32_t s = lo;
  const int32_t cu_s = p.cu_new_lens[s];
  const int32_t i = tok - cu_s;
  const int32_t P = p.prefix_lens[s];
  const int32_t G = p.n_q_heads / p.n_kv_heads;
  const int32_t g = h / G;
  const int32_t n_keys = P + i + 1;

  const T* q = (const T*)p.q + ((int64_t)tok * p.n_q_heads + h) * D;
  for (int c = lane; c < D; c += 64) q_s[c] = to_f32(q[c]);
  __syncthreads();

  float m = -INFINITY, l = 0.f;
  float acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.f;

  for (int32_t j = lane; j < n_keys; j += 64) {
    const T* kp;
    const T* vp;
    if (j < P) {
      const int32_t jb = j / p.block_size;
      const int32_t b = jb < p.table_stride ? p.table[(int64_t)s * p.table_stride + jb] : -1;
      if (b < 0 || b >= p.n_blocks) continue;
      const int64_t e = (int64_t)b * p.block_stride + ((int64_t)(j - jb * p.block_size) * p.n_kv_heads + g) * D;
      kp = (const T*)p.k_layer + e;
      vp = (const T*)p.v_layer + e;
    } else {
      const int64_t e = ((int64_t)(cu_s + j - P) * p.n_kv_heads + g) * D;
      kp = (const T*)p.k_new + e;
      vp = (const T*)p.v_new + e;
    }
    float dot = 0.f;
#pragma unroll 8
    for (int c = 0; c < D; ++c) dot = fmaf(q_s[c], to_f32(kp[c]), dot);
    const float x = p.scale * dot;
    const float m_new = fmaxf(m, x);
    const float alpha = expf(m - m_new);  // m = -inf on the first key: alpha = 0
    const float w = expf(x - m_new);
    l = l * alpha + w;
#pragma unroll
    for (int c = 0; c < D; ++c) acc[c] = fmaf(w, to_f32(vp[c]), acc[c] * alpha);
    m = m_new;
  }

  // merge the 64 per-lane partial softmaxes
  float M = m;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  const float f = (m == -INFINITY) ? 0.f : expf(m - M);
  float lt = l * f;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) lt += __shfl_xor(lt, o);
  const float inv = 1.0f / lt;
  T* out = (T*)p.out + ((int64_t)tok * p.n_q_heads + h) * D;
#pragma unroll
  for (int c = 0; c < D; ++c) {
    float a = acc[c] * f;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) a += __shfl_xor(a, o);
    if (lane == (c & 63)) from_f32(out + c, a * inv);
  }
}

// ------------------------------------------------------------------------------------------------------------
// bf16 MFMA path, head_dim 128
// ------------------------------------------------------------------------------------------------------------
// Work decomposition.  A "unit" is (session, tile of BMT = 128/G query tokens); its cost is the number of 64-key
// tiles it has to visit.  A scheduling kernel (one workgroup) turns the ragged batch into a list of work items:
// units longer than a chunk length C are split along the key axis into near-equal chunks (C is chosen so that the
// batch gives about `target` workgroup-sized pieces), and the items are ordered longest first, so that the
// hardware's in-order workgroup dispatch is a longest-processing-time list schedule.  Every item is executed for
// every kv-head by one workgroup: global index g -> (item g / H_kv, kv-head g % H_kv), which with 8 kv-heads also
// pins each kv-head to one XCD (workgroups are dealt round-robin to the 8 XCDs), so the query tiles of a session
// that re-read the same K,V share that XCD's L2.  Chunks of a split unit write unnormalised partial results
// (running max, running sum, accumulators) to the workspace and a merge kernel combines them.
struct WorkItem {   // 32 bytes
  int32_t s, t0, tile_begin, tile_end, pslot, pad0, pad1, pad2;   // pslot < 0: whole unit, write the output directly
};
struct MergeItem {  // 16 bytes
  int32_t s, t0, pslot0, n_chunks;
};
constexpr int kHdrInts = 64;
constexpr int kPartialFloats = 256 * 66;  // per workgroup: 64 accumulators + running max + running sum per thread

struct SchedParams {
  const int32_t* cu_new_lens;
  const int32_t* prefix_lens;
  int32_t n_sessions, bmt, n_kv_heads, target, c_min;
  int32_t items_bound, merges_bound, pslots_bound;
  int32_t* hdr;
  WorkItem* items;
  MergeItem* merges;
};

constexpr int kBN = 64;  // keys per tile
constexpr int kSchedThreads = 1024;
constexpr int kSchedBuckets = 1024;

__device__ __forceinline__ int unit_tiles(int P, int N, int t0, int bmt) {
  return (P + min(N, t0 + bmt) + kBN - 1) / kBN;
}

__global__ __launch_bounds__(kSchedThreads) void attn_schedule_kernel(const SchedParams p) {
  __shared__ unsigned long long total_tiles_s;
  __shared__ int hist[kSchedBuckets];
  __shared__ int n_items_s, n_merge_s, n_pslot_s, chunk_s;
  const int tid = threadIdx.x;
  if (tid == 0) {
    total_tiles_s = 0ull;
    n_items_s = 0;
    n_merge_s = 0;
    n_pslot_s = 0;
  }
  for (int b = tid; b < kSchedBuckets; b += kSchedThreads) hist[b] = 0;
  __syncthreads();
  // pass 1: total number of (unit, key tile) pairs
  unsigned long long mine = 0;
  for (int s = tid; s < p.n_sessions; s += kSchedThreads) {
    const int N = p.cu_new_lens[s + 1] - p.cu_new_lens[s];
    const int P = p.prefix_lens[s];
    for (int t0 = 0; t0 < N; t0 += p.bmt) mine += (unsigned long long)unit_tiles(P, N, t0, p.bmt);
  }
  if (mine) atomicAdd(&total_tiles_s, mine);
  __syncthreads();
  if (tid == 0) {
    const unsigned long long tot = total_tiles_s * (unsigned long long)p.n_kv_heads;
    long long c = (long long)((tot + p.target - 1) / (unsigned long long)p.target);
    if (c < p.c_min) c = p.c_min;
    if (c > 0x3FFFFFFF) c = 0x3FFFFFFF;
    chunk_s = (int)c;
  }
  __syncthreads();
  const int C = chunk_s;
  // bucket of a chunk length len in 1..C: longer chunks get smaller bucket numbers (they are dispatched first)
  auto bucket_of = [&](int len) {
    long long b = (long long)(C - len) * kSchedBuckets / C;
    return (int)(b < 0 ? 0 : (b >= kSchedBuckets ? kSchedBuckets - 1 : b));
  };
  // pass 2: histogram of chunk lengths
  for (int s = tid; s < p.n_sessions; s += kSchedThreads) {
    const int N = p.cu_new_lens[s + 1] - p.cu_new_lens[s];
    const int P = p.prefix_lens[s];
    for (int t0 = 0; t0 < N; t0 += p.bmt) {
      const int nt = unit_tiles(P, N, t0, p.bmt);
      const int nc = (nt + C - 1) / C;
      const int len = (nt + nc - 1) / nc;
      for (int ch = 0; ch < nc; ++ch) {
        const int tb = ch * len, te = min(nt, tb + len);
        if (te > tb) atomicAdd(&hist[bucket_of(te - tb)], 1);
      }
    }
  }
  __syncthreads();
  if (tid == 0) {  // exclusive prefix sum: hist[b] becomes the first list position of bucket b
    int run = 0;
    for (int b = 0; b < kSchedBuckets; ++b) {
      const int h = hist[b];
      hist[b] = run;
      run += h;
    }
    n_items_s = run;
  }
  __syncthreads();
  // pass 3: emit items
  for (int s = tid; s < p.n_sessions; s += kSchedThreads) {
    const int N = p.cu_new_lens[s + 1] - p.cu_new_lens[s];
    const int P = p.prefix_lens[s];
    for (int t0 = 0; t0 < N; t0 += p.bmt) {
      const int nt = unit_tiles(P, N, t0, p.bmt);
      const int nc = (nt + C - 1) / C;
      const int len = (nt + nc - 1) / nc;
      int n_real = 0;
      for (int ch = 0; ch < nc; ++ch)
        if (min(nt, (ch + 1) * len) > ch * len) ++n_real;
      int pslot0 = -1;
      if (n_real > 1) {
        pslot0 = atomicAdd(&n_pslot_s, n_real);
        const int mi = atomicAdd(&n_merge_s, 1);
        if (mi < p.merges_bound && pslot0 + n_real <= p.pslots_bound) {
          p.merges[mi] = MergeItem{s, t0, pslot0, n_real};
        } else {
          pslot0 = -2;  // cannot happen while the host-side bounds hold; fall back to not emitting the unit
        }
      }
      if (pslot0 == -2) continue;
      int k = 0;
      for (int ch = 0; ch < nc; ++ch) {
        const int tb = ch * len, te = min(nt, tb + len);
        if (te <= tb) continue;
        const int pos = atomicAdd(&hist[bucket_of(te - tb)], 1);
        if (pos < p.items_bound) p.items[pos] = WorkItem{s, t0, tb, te, pslot0 < 0 ? -1 : pslot0 + k, 0, 0, 0};
        ++k;
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    p.hdr[0] = min(n_items_s, p.items_bound);
    p.hdr[1] = C;
    p.hdr[2] = min(n_merge_s, p.merges_bound);
    p.hdr[3] = n_pslot_s;
  }
}

struct MfmaParams {
  const __bf16* k_layer;
  const __bf16* v_layer;
  int64_t block_stride;
  uint32_t block_bytes;  // block_stride in bytes (the MFMA path requires it to fit 32 bits)
  uint32_t row_bytes;    // one token row of K (or V): n_kv_heads * 128 * 2
  int32_t n_blocks, log_bs, n_kv_heads, n_q_heads;
  const __bf16* q;
  const __bf16* k_new;
  const __bf16* v_new;
  __bf16* out;
  const int32_t* cu_new_lens;
  const int32_t* prefix_lens;
  const int32_t* table;
  int32_t table_stride, n_sessions;
  float scale_log2e;
  const int32_t* hdr;
  const WorkItem* items;
  const MergeItem* merges;
  float* partials;
};

constexpr int kD = 128;         // head_dim
constexpr int kKsStride = 136;  // bf16 per K row in LDS: 272 B, so 16-byte reads of 16 different rows cover all banks
constexpr int kVsStride = 160;  // bf16 per V row in LDS: 320 B, so the 4 rows of a transposing read are 16 banks apart

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// Row r (0..31) of the A operand of S^T = K Q^T holds key key_of_row(r) of the 32-key block, chosen so that the
// MFMA result registers 8*u .. 8*u+7 of a lane in half-wave g2 are keys 16*u + 8*g2 + 0..7.
__device__ __forceinline__ int key_of_row(int r) {
  const int j = r & 3, gg = (r >> 2) & 1, i = r >> 3;
  return 16 * (i >> 1) + 8 * gg + 4 * (i & 1) + j;
}

// ds_read_b64_tr_b16: the 16 lanes of a group hand in the addresses of a 4 x 16 tile of 16-bit values (lanes
// 4e .. 4e+3 cover row e, 4 values each) and lane i gets column i, i.e. 4 consecutive rows of one column.
__device__ __forceinline__ s16x4 lds_read_tr16(const __bf16* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(const_cast<__bf16*>(p)));
}

// Write one query row's 128 outputs: this lane holds d = 32*dt + 4*g2 + 8*i + j at acc[dt][4*i + j].
__device__ __forceinline__ void store_out_row(__bf16* op, const f32x16 (&acc)[4], float inv, int g2) {
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x4 v;
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = (__bf16)(acc[dt][4 * i + j] * inv);
      *reinterpret_cast<bf16x4*>(op + 32 * dt + 4 * g2 + 8 * i) = v;
    }
}

// Lanes l and l^32 hold the two halves of one query's keys.  v_permlane32_swap_b32 a, b exchanges lanes 32..63 of a
// with lanes 0..31 of b, so starting from two copies of x it leaves a = low half twice, b = high half twice.
// Written as inline assembly: with this compiler the builtin hands back the first register for both results.
__device__ __forceinline__ void swap_halves(float x, float& lo_twice, float& hi_twice) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  lo_twice = a;
  hi_twice = b;
}
__device__ __forceinline__ float max_across_halves(float x) {
  float lo, hi;
  swap_halves(x, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_across_halves(float x) {
  float lo, hi;
  swap_halves(x, lo, hi);
  return lo + hi;
}

constexpr int kKsElems = kBN * kKsStride;
constexpr int kVsElems = kBN * kVsStride;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// One workgroup = one work item x one kv-head: 128 query rows (G heads x 128/G tokens) against the item's key tiles.
// Requires block_size >= 16 (a power of two): the 16 consecutive key rows that a group of 16 threads stages then lie
// in ONE block, so block ids are workgroup-uniform, live in scalar registers, and a row address is
// scalar base + per-thread constant.  LB = log2(block_size) when it is 4 (the common 16-token block), else 0 = runtime.
//
// Each wave issues at most one instruction every four cycles, so the loop over key tiles is written for a low
// instruction count: tiles that lie wholly inside the paged prefix run through a loop that is unrolled twice (one
// copy per LDS buffer, all LDS offsets immediate, no masking, no per-row bounds logic); the few tiles around the
// prefix / new-turn boundary and the causal diagonal take a general path.
template <int G, int LB>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(const MfmaParams p) {
  constexpr int BMT = 128 / G;  // query tokens per tile
  __shared__ __attribute__((aligned(16))) __bf16 Ks[2 * kKsElems];  // double-buffered K tile [64 keys][128 d]
  __shared__ __attribute__((aligned(16))) __bf16 Vs[2 * kVsElems];  // double-buffered V tile [64 keys][128 d]

  const int Hkv = p.n_kv_heads;
  const int item_idx = blockIdx.x / Hkv;
  if (item_idx >= p.hdr[0]) return;
  const int kvh = blockIdx.x - item_idx * Hkv;
  const WorkItem it = p.items[item_idx];
  const int s = it.s;
  const int t0 = it.t0;
  const int cu_s = p.cu_new_lens[s];
  const int N = p.cu_new_lens[s + 1] - cu_s;
  const int P = p.prefix_lens[s];
  const int lb = LB ? LB : p.log_bs;
  const int bs_mask = (1 << lb) - 1;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int n = lane & 31;  // query column of this lane inside the wave's 32 rows; also its A-operand row
  const int g2 = lane >> 5;

  // query row of this lane: head-major inside the tile
  const int r = wave * 32 + n;
  const int hh = r / BMT;
  const int tt = r - hh * BMT;
  const int tok = t0 + tt;
  const bool q_valid = tok < N;
  const int head = kvh * G + hh;

  bf16x8 qreg[8];
  {
    const __bf16* qp = p.q + ((int64_t)(cu_s + (q_valid ? tok : 0)) * p.n_q_heads + head) * kD + 8 * g2;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      qreg[st] = *reinterpret_cast<const bf16x8*>(qp + 16 * st);
      if (!q_valid) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qreg[st][e] = (__bf16)0.0f;
      }
    }
  }

  const int total_keys = P + N;
  const int tile_begin = it.tile_begin, tile_end = it.tile_end;
  // tiles below fast_end lie entirely inside the paged prefix: every row comes from the pool, nothing is masked
  const int fast_end = min(tile_end, P / kBN);

  // staging map: thread -> 16-byte chunk c of key rows kr, kr+16, kr+32, kr+48 of the tile
  const int c = tid & 15;
  const int kr = tid >> 4;
  const bool has_table = p.table != nullptr && p.table_stride > 0;
  const int32_t* table_row = p.table + (int64_t)s * p.table_stride;
  const int row_elems = Hkv * kD;
  const int thr_off = kvh * kD + 8 * c;                              // offset inside a token row (elements)
  const unsigned voff = (unsigned)(kr * row_elems + thr_off) * 2u;   // byte offset from a 16-row group's base
  const char* k_bytes = reinterpret_cast<const char*>(p.k_layer);
  const char* v_bytes = reinterpret_cast<const char*>(p.v_layer);

  // Block ids of the tile's four 16-row groups (scalar registers), loaded one tile ahead of the K,V rows themselves so
  // that the two dependent global reads never sit on the critical path.
  int ids[4];
  auto load_ids = [&](int tile) {
    if (has_table) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int jb = (tile * kBN + 16 * i) >> lb;
        ids[i] = __builtin_amdgcn_readfirstlane(table_row[min(jb, p.table_stride - 1)]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) ids[i] = -1;
    }
  };
  u32x4 kreg[4], vreg[4];
  unsigned okbits = 0xF;  // bit i: the rows of group i that this thread staged exist (uniform for fast tiles)
  auto fetch_fast = [&](int tile) {
    unsigned ok = 0xF;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned b = (unsigned)ids[i];
      const unsigned bc = min(b, (unsigned)(p.n_blocks - 1));  // out-of-range ids are never dereferenced
      if (bc != b) ok &= ~(1u << i);
      uint64_t off = (uint64_t)bc * p.block_bytes;
      if (LB != 4) off += (uint64_t)((tile * kBN + 16 * i) & bs_mask) * p.row_bytes;
      kreg[i] = *reinterpret_cast<const u32x4*>(k_bytes + off + voff);
      vreg[i] = *reinterpret_cast<const u32x4*>(v_bytes + off + voff);
    }
    okbits = ok;
  };
  auto fetch_general = [&](int tile) {  // unconditional loads (a safe dummy address for absent rows), zeroed when staged
    unsigned ok = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = tile * kBN + 16 * i + kr;
      const int b = ids[i];
      const bool in_pool = key < P && (key >> lb) < p.table_stride && (unsigned)b < (unsigned)p.n_blocks;
      const bool in_new = key >= P && key < total_keys;
      const int64_t e_pool = (int64_t)(in_pool ? b : 0) * p.block_stride + (key & bs_mask) * row_elems + thr_off;
      const int64_t e_new = (int64_t)(cu_s + key - P) * row_elems + thr_off;
      const __bf16* kp = in_pool ? p.k_layer + e_pool : (in_new ? p.k_new + e_new : p.q);
      const __bf16* vp = in_pool ? p.v_layer + e_pool : (in_new ? p.v_new + e_new : p.q);
      kreg[i] = *reinterpret_cast<const u32x4*>(kp);
      vreg[i] = *reinterpret_cast<const u32x4*>(vp);
      if (in_pool || in_new) ok |= 1u << i;
    }
    okbits = ok;
  };
  __bf16* const k_wr = Ks + kr * kKsStride + 8 * c;
  __bf16* const v_wr = Vs + kr * kVsStride + 8 * c;
  auto stage = [&](int buf) {
    __bf16* ks = k_wr + buf * kKsElems;
    __bf16* vs = v_wr + buf * kVsElems;
    if (okbits == 0xF) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<u32x4*>(ks + 16 * i * kKsStride) = kreg[i];
        *reinterpret_cast<u32x4*>(vs + 16 * i * kVsStride) = vreg[i];
      }
    } else {
      const u32x4 z = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<u32x4*>(ks + 16 * i * kKsStride) = (okbits >> i) & 1 ? kreg[i] : z;
        *reinterpret_cast<u32x4*>(vs + 16 * i * kVsStride) = (okbits >> i) & 1 ? vreg[i] : z;
      }
    }
  };

  f32x16 o_acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o_acc[dt][e] = 0.f;
  float m_run = -INFINITY;  // running max of raw scores (before scale)
  float l_run = 0.f;        // this lane's share of the running sum
  const float cs = p.scale_log2e;
  const int q_limit = P + tok;  // last key this query may see
  const __bf16* const k_rd = &Ks[key_of_row(n) * kKsStride + 8 * g2];
  // transposing V read: lane group (lane/16) = 2*g2 + dhalf reads rows (keys) 8*g2 + i16/4 (+4), columns
  // 16*dhalf + 4*(i16%4) .. +3 and receives, for column d = 16*dhalf + i16, four consecutive keys
  const int i16 = lane & 15;
  const __bf16* const v_rd = &Vs[(8 * g2 + (i16 >> 2)) * kVsStride + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3)];
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  // One key tile: S^T = K Q^T, online softmax (one query per lane), O^T += V^T P^T.  MASKED: the tile may reach past
  // some query's causal limit, or the work item may start past it (then a row may have seen no key at all yet).
  auto compute = [&](const __bf16* k_cur, const __bf16* v_cur, int tile, auto masked_c) {
    constexpr bool MASKED = decltype(masked_c)::value;
    f32x16 sc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) sc[kb][e] = 0.f;
    if (!(SYMPH_DEV_ABLATE & 8)) {
      // K fragments of the second 32-key block are read while the first block multiplies
      bf16x8 ka[8];
#pragma unroll
      for (int st = 0; st < 8; ++st) ka[st] = *reinterpret_cast<const bf16x8*>(k_cur + 16 * st);
#pragma unroll
      for (int st = 0; st < 8; ++st) {
        sc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[st], qreg[st], sc[0], 0, 0, 0);
        ka[st] = *reinterpret_cast<const bf16x8*>(k_cur + 32 * kKsStride + 16 * st);
      }
#pragma unroll
      for (int st = 0; st < 8; ++st) sc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[st], qreg[st], sc[1], 0, 0, 0);
    }
    if (MASKED) {
      const int key0 = tile * kBN;
      if (key0 + kBN - 1 > P + t0) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int key = key0 + kb * 32 + 16 * (e >> 3) + 8 * g2 + (e & 7);
            if (key > q_limit) sc[kb][e] = -INFINITY;
          }
      }
    }
    // online softmax; two lanes, l and l^32, share a query and split its keys
    float mx = sc[0][0];
    if (!(SYMPH_DEV_ABLATE & 1)) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[kb][e]);
      mx = max_across_halves(mx);
    }
    const float m_new = fmaxf(m_run, mx);
    // a row that has seen no key yet (possible only on the MASKED path) keeps its exponent arguments finite
    const float m_use = (MASKED && m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * cs);
    const float mb = m_use * cs;
    bf16x8 pb[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pv = (SYMPH_DEV_ABLATE & 1) ? sc[kb][e] : __builtin_amdgcn_exp2f(fmaf(sc[kb][e], cs, -mb));
        pb[kb][e >> 3][e & 7] = (__bf16)pv;
      }
    // row sum of the ROUNDED probabilities (the values the second product uses), two per instruction
    float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 v = pb[kb][u];
        ps0 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[0], v[1]}, ones, ps0, false);
        ps1 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[2], v[3]}, ones, ps1, false);
        ps0 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[4], v[5]}, ones, ps0, false);
        ps1 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[6], v[7]}, ones, ps1, false);
      }
    l_run = fmaf(l_run, alpha, ps0 + ps1);
    if (__any(m_new != m_run)) {  // the running max moved for some query of this wave: rescale the accumulators
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[dt][e] *= alpha;
    }
    m_run = m_new;
    if (SYMPH_DEV_ABLATE & 4) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int u = 0; u < 2; ++u) o_acc[kb][u] += (float)pb[kb][u][0] + (float)pb[kb][u][7];
    } else {
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const __bf16* vp = v_cur + (kb * 32 + 16 * u) * kVsStride + 32 * dt;
            const s16x4 lo = lds_read_tr16(vp);
            const s16x4 hi = lds_read_tr16(vp + 4 * kVsStride);
            const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb[kb][u], o_acc[dt],
                                                                0, 0, 0);
          }
    }
  };

  // prologue: tile_begin staged in buffer 0, tile_begin+1 in flight, ids of tile_begin+2 loaded
  auto fetch = [&](int tile) {
    if (tile < fast_end)
      fetch_fast(tile);
    else
      fetch_general(tile);
  };
  load_ids(tile_begin);
  fetch(tile_begin);
  if (tile_begin + 1 < tile_end) load_ids(tile_begin + 1);
  stage(0);
  if (tile_begin + 1 < tile_end) {
    fetch(tile_begin + 1);
    if (tile_begin + 2 < tile_end) load_ids(tile_begin + 2);
  }
  __syncthreads();

  int tile = tile_begin;
  // fast loop: while tiles tile .. tile+3 all lie inside the paged prefix, two iterations per trip (buffers 0 and 1).
  // Iteration t computes tile t from one buffer, stages tile t+1 into the other, fetches tile t+2, loads ids of t+3.
  if (!(SYMPH_DEV_ABLATE & 2)) {
    while (tile + 3 < fast_end) {
      stage(1);
      fetch_fast(tile + 2);
      load_ids(tile + 3);
      compute(k_rd, v_rd, tile, std::false_type{});
      __syncthreads();
      stage(0);
      fetch_fast(tile + 3);
      load_ids(tile + 4);
      compute(k_rd + kKsElems, v_rd + kVsElems, tile + 1, std::false_type{});
      __syncthreads();
      tile += 2;
    }
  }
  // general loop: boundary and diagonal tiles (and any leftover fast tile)
  for (; tile < tile_end; ++tile) {
    const int cur = (tile - tile_begin) & 1;
    if (tile + 1 < tile_end && !(SYMPH_DEV_ABLATE & 2)) {  // the other buffer was last read before the last barrier
      stage(cur ^ 1);
      if (tile + 2 < tile_end) {
        fetch(tile + 2);
        if (tile + 3 < tile_end) load_ids(tile + 3);
      }
    }
    const int rb = (SYMPH_DEV_ABLATE & 2) ? 0 : cur;
    compute(k_rd + rb * kKsElems, v_rd + rb * kVsElems, tile, std::true_type{});
    __syncthreads();
  }

  if (it.pslot < 0) {
    const float l_tot = sum_across_halves(l_run);
    if (q_valid)
      store_out_row(p.out + ((int64_t)(cu_s + tok) * p.n_q_heads + head) * kD, o_acc, 1.0f / l_tot, g2);
  } else {
    // register dump, one float per thread per store: fully coalesced, and the merge kernel uses the same mapping
    float* part = p.partials + ((int64_t)it.pslot * Hkv + kvh) * kPartialFloats + tid;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) part[(dt * 16 + e) * 256] = o_acc[dt][e];
    part[64 * 256] = m_run;
    part[65 * 256] = l_run;
  }
}

// Combine the chunks of a split unit: out = sum_c w_c O_c / sum_c w_c l_c with w_c = 2^((m_c - max_c m_c) * cs).
template <int G>
__global__ __launch_bounds__(256) void attn_merge_kernel(const MfmaParams p) {
  constexpr int BMT = 128 / G;
  const int Hkv = p.n_kv_heads;
  const int mi = blockIdx.x / Hkv;
  if (mi >= p.hdr[2]) return;
  const int kvh = blockIdx.x - mi * Hkv;
  const MergeItem m = p.merges[mi];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int n = lane & 31, g2 = lane >> 5;
  const int r = (tid >> 6) * 32 + n;
  const int hh = r / BMT;
  const int tok = m.t0 + (r - hh * BMT);
  const int cu_s = p.cu_new_lens[m.s];
  const int N = p.cu_new_lens[m.s + 1] - cu_s;
  const float cs = p.scale_log2e;
  const float* base = p.partials + ((int64_t)m.pslot0 * Hkv + kvh) * kPartialFloats + tid;
  const int64_t chunk_stride = (int64_t)Hkv * kPartialFloats;
  float M = -INFINITY;
  for (int ch = 0; ch < m.n_chunks; ++ch) M = fmaxf(M, base[ch * chunk_stride + 64 * 256]);
  f32x16 acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[dt][e] = 0.f;
  float L = 0.f;
  for (int ch = 0; ch < m.n_chunks; ++ch) {
    const float* part = base + ch * chunk_stride;
    const float mc = part[64 * 256];
    const float w = (mc == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((mc - M) * cs);
    L += w * part[65 * 256];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[dt][e] = fmaf(w, part[(dt * 16 + e) * 256], acc[dt][e]);
  }
  const float l_tot = sum_across_halves(L);
  if (tok < N)
    store_out_row(p.out + ((int64_t)(cu_s + tok) * p.n_q_heads + (kvh * G + hh)) * kD, acc, 1.0f / l_tot, g2);
}

// ------------------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------------------
static int env_int(const char* name, int dflt) {
  const char* e = getenv(name);
  return e ? atoi(e) : dflt;
}

struct MfmaPlan {
  int32_t bmt, target, c_min, units_bound, items_bound, merges_bound, pslots_bound;
  int64_t off_items, off_merges, off_partials, total_bytes;
};

static inline int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

// Sizes that depend only on host-visible bounds, so that the workspace query and the launch agree.
static MfmaPlan make_plan(int32_t n_sessions, int32_t n_q_heads, int32_t n_kv_heads, int32_t total_new_tokens) {
  MfmaPlan pl;
  const int G = n_q_heads / n_kv_heads;
  pl.bmt = 128 / G;
  pl.target = env_int("SYMPH_ATTN_TARGET", 1024);  // workgroup-sized pieces the batch is cut into (about 2 per slot)
  if (pl.target < n_kv_heads) pl.target = n_kv_heads;
  pl.c_min = env_int("SYMPH_ATTN_CMIN", 8);
  if (pl.c_min < 1) pl.c_min = 1;
  pl.units_bound = total_new_tokens / pl.bmt + n_sessions;
  const int32_t per_head = pl.target / n_kv_heads + 1;
  pl.items_bound = pl.units_bound + per_head;
  pl.merges_bound = per_head;
  pl.pslots_bound = 2 * per_head;
  pl.off_items = align256(kHdrInts * 4);
  pl.off_merges = align256(pl.off_items + (int64_t)pl.items_bound * sizeof(WorkItem));
  pl.off_partials = align256(pl.off_merges + (int64_t)pl.merges_bound * sizeof(MergeItem));
  pl.total_bytes = pl.off_partials + (int64_t)pl.pslots_bound * n_kv_heads * kPartialFloats * 4;
  return pl;
}

static bool mfma_path_ok(int32_t dtype, int32_t head_dim, int32_t n_q_heads, int32_t n_kv_heads, int32_t block_size) {
  if (dtype != SYMPH_BF16 || head_dim != 128) return false;
  const int G = n_q_heads / n_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16) return false;
  return block_size >= 16 && (block_size & (block_size - 1)) == 0;
}

int64_t prefill_attn_workspace_bytes(const symph_kv_cache* c, int32_t n_sessions, int32_t n_q_heads,
                                     int32_t total_new_tokens, int32_t, int32_t) {
  if (n_q_heads % c->n_kv_heads != 0) return -1;
  if (!mfma_path_ok(c->dtype, c->head_dim, n_q_heads, c->n_kv_heads, c->block_size)) return 0;
  return make_plan(n_sessions, n_q_heads, c->n_kv_heads, total_new_tokens).total_bytes;
}

template <typename T, int D>
static int32_t launch_generic(const AttnArgs& a, hipStream_t stream) {
  GenericParams p;
  p.k_layer = a.k_layer;
  p.v_layer = a.v_layer;
  p.block_stride = a.block_stride;
  p.n_blocks = a.n_blocks;
  p.block_size = a.block_size;
  p.n_kv_heads = a.n_kv_heads;
  p.n_q_heads = a.n_q_heads;
  p.q = a.q;
  p.k_new = a.k_new;
  p.v_new = a.v_new;
  p.out = a.out;
  p.cu_new_lens = a.cu_new_lens;
  p.prefix_lens = a.prefix_lens;
  p.table = a.table;
  p.table_stride = a.table_stride;
  p.n_sessions = a.n_sessions;
  p.total_new_tokens = a.total_new_tokens;
  p.scale = a.scale;
  const int64_t rows = (int64_t)a.total_new_tokens * a.n_q_heads;
  if (rows > 0x7FFFFFFFLL) return SYMPH_EUNSUPPORTED;
  hipLaunchKernelGGL((attn_generic_kernel<T, D>), dim3((unsigned)rows), dim3(64), 0, stream, p);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

template <int G>
static int32_t launch_mfma(const AttnArgs& a, hipStream_t stream) {
  const MfmaPlan pl = make_plan(a.n_sessions, a.n_q_heads, a.n_kv_heads, a.total_new_tokens);
  if (!a.workspace || a.workspace_bytes < pl.total_bytes) return SYMPH_EWORKSPACE;
  if (((uintptr_t)a.workspace & 255) != 0) return SYMPH_EUNSUPPORTED;
  char* ws = (char*)a.workspace;

  SchedParams sp;
  sp.cu_new_lens = a.cu_new_lens;
  sp.prefix_lens = a.prefix_lens;
  sp.n_sessions = a.n_sessions;
  sp.bmt = pl.bmt;
  sp.n_kv_heads = a.n_kv_heads;
  sp.target = pl.target;
  sp.c_min = pl.c_min;
  sp.items_bound = pl.items_bound;
  sp.merges_bound = pl.merges_bound;
  sp.pslots_bound = pl.pslots_bound;
  sp.hdr = (int32_t*)ws;
  sp.items = (WorkItem*)(ws + pl.off_items);
  sp.merges = (MergeItem*)(ws + pl.off_merges);

  MfmaParams p;
  p.k_layer = (const __bf16*)a.k_layer;
  p.v_layer = (const __bf16*)a.v_layer;
  p.block_stride = a.block_stride;
  p.block_bytes = (uint32_t)(a.block_stride * 2);
  p.row_bytes = (uint32_t)a.n_kv_heads * kD * 2u;
  p.n_blocks = a.n_blocks;
  p.log_bs = __builtin_ctz((unsigned)a.block_size);
  p.n_kv_heads = a.n_kv_heads;
  p.n_q_heads = a.n_q_heads;
  p.q = (const __bf16*)a.q;
  p.k_new = (const __bf16*)a.k_new;
  p.v_new = (const __bf16*)a.v_new;
  p.out = (__bf16*)a.out;
  p.cu_new_lens = a.cu_new_lens;
  p.prefix_lens = a.prefix_lens;
  p.table = a.table;
  p.table_stride = a.table_stride;
  p.n_sessions = a.n_sessions;
  p.scale_log2e = a.scale * 1.4426950408889634f;
  p.hdr = sp.hdr;
  p.items = sp.items;
  p.merges = sp.merges;
  p.partials = (float*)(ws + pl.off_partials);

  const int64_t g_main = (int64_t)pl.items_bound * a.n_kv_heads;
  const int64_t g_merge = (int64_t)pl.merges_bound * a.n_kv_heads;
  if (g_main > 0x7FFFFFFFLL) return SYMPH_EUNSUPPORTED;
  hipLaunchKernelGGL(attn_schedule_kernel, dim3(1), dim3(kSchedThreads), 0, stream, sp);
  if (a.block_size == 16)
    hipLaunchKernelGGL((attn_mfma_kernel<G, 4>), dim3((unsigned)g_main), dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL((attn_mfma_kernel<G, 0>), dim3((unsigned)g_main), dim3(256), 0, stream, p);
  hipLaunchKernelGGL((attn_merge_kernel<G>), dim3((unsigned)g_merge), dim3(256), 0, stream, p);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

int32_t launch_prefill_attn(const AttnArgs& a, hipStream_t stream) {
  const int G = a.n_q_heads / a.n_kv_heads;
  const bool aligned16 = (((uintptr_t)a.k_layer | (uintptr_t)a.v_layer | (uintptr_t)a.q | (uintptr_t)a.k_new |
                           (uintptr_t)a.v_new | (uintptr_t)a.out | (uintptr_t)(a.block_stride * 2)) & 15) == 0;
  if (mfma_path_ok(a.dtype, a.head_dim, a.n_q_heads, a.n_kv_heads, a.block_size) &&
      a.block_stride * 2 <= 0xFFFFFFFFLL) {
    if (!aligned16) return SYMPH_EUNSUPPORTED;
    switch (G) {
      case 1: return launch_mfma<1>(a, stream);
      case 2: return launch_mfma<2>(a, stream);
      case 4: return launch_mfma<4>(a, stream);
      case 8: return launch_mfma<8>(a, stream);
      case 16: return launch_mfma<16>(a, stream);
      default: break;
    }
  }
  if (a.dtype == SYMPH_BF16) {
    if (a.head_dim == 64) return launch_generic<__bf16, 64>(a, stream);
    if (a.head_dim == 128) return launch_generic<__bf16, 128>(a, stream);
  } else {
    if (a.head_dim == 64) return launch_generic<float, 64>(a, stream);
    if (a.head_dim == 128) return launch_generic<float, 128>(a, stream);
  }
  return SYMPH_EUNSUPPORTED;
}

}  // namespace symph
