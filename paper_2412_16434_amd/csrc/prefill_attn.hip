// prefix_prefill_attn: the new turn's GQA queries against [paged cached prefix ; causal new tokens]
// (Symphony Sec. 2.1: A_h = softmax(Q_h K_h^T * scale), y = concat_h A_h V_h; a token sees all prior tokens).
//
// bf16 path (head_dim 128), one workgroup of 4 waves per (session, kv-head, tile of query tokens):
//   * the G query heads that share a kv-head are stacked into the tile (128 query rows = G heads x 128/G tokens),
//     so every K,V tile staged in LDS is reused by all of them;
//   * scores are computed TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: the MFMA result layout then puts
//     one query per lane, so the online-softmax state (reference, running sum) is per-lane scalars, and the bf16
//     probabilities a lane holds are exactly the B operand of O^T += V^T P^T;
//   * the row order in which K rows are fed to the MFMA is permuted so that the 8 probabilities a lane needs for
//     one 16-key step of the second product are 8 consecutive keys; the matching V^T operand comes from the
//     transposing LDS read (ds_read_b64_tr_b16), V stays row-major in LDS;
//   * K,V tiles of 64 keys go from the paged pool (block-table indirection per 16-token block) or from the
//     contiguous new-turn K,V straight into LDS (global_load_lds_dwordx4), double-buffered, one tile ahead;
//   * the softmax reference is stale on purpose (refreshed only when a row sum shows that it has to be), so no
//     per-tile maximum and no per-tile rescaling of the accumulators.
// generic path (fp32, or head_dim 64): one wave per query row, lanes over keys, fp32 online softmax.
#include "common.h"

#include <type_traits>

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
    const T* kp = nullptr;  // a block id outside the cache names a row of zeros (score 0, value 0), as in the MFMA path
    const T* vp = nullptr;
    if (j < P) {
      const int32_t jb = j / p.block_size;
      const int32_t b = jb < p.table_stride ? p.table[(int64_t)s * p.table_stride + jb] : -1;
      if (b >= 0 && b < p.n_blocks) {
        const int64_t e = (int64_t)b * p.block_stride + ((int64_t)(j - jb * p.block_size) * p.n_kv_heads + g) * D;
        kp = (const T*)p.k_layer + e;
        vp = (const T*)p.v_layer + e;
      }
    } else {
      const int64_t e = ((int64_t)(cu_s + j - P) * p.n_kv_heads + g) * D;
      kp = (const T*)p.k_new + e;
      vp = (const T*)p.v_new + e;
    }
    float dot = 0.f;
    if (kp) {
#pragma unroll 8
      for (int c = 0; c < D; ++c) dot = fmaf(q_s[c], to_f32(kp[c]), dot);
    }
    const float x = p.scale * dot;
    const float m_new = fmaxf(m, x);
    const float alpha = expf(m - m_new);  // m = -inf on the first key: alpha = 0
    const float w = expf(x - m_new);
    l = l * alpha + w;
    if (vp) {
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = fmaf(w, to_f32(vp[c]), acc[c] * alpha);
    } else {
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] *= alpha;
    }
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
  const float inv = lt > 0.f ? 1.0f / lt : 0.f;  // (every row sees at least itself, so the sum is positive)
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
struct WorkItem {   // 96 bytes
  int32_t s, t0, tile_begin, tile_end;
  int32_t pslot;                  // < 0: whole unit, the workgroup writes the output rows itself
  int32_t cu_s, n_new, n_prefix;  // of session s, so that a workgroup starts without looking them up
  int32_t merge, pslot0, n_chunks;  // chunk of a split unit: the unit's counter, its first slot, its number of chunks
  int32_t first_ids[8];           // block ids of the eight 16-key groups of tiles tile_begin and tile_begin + 1: the
                                  // workgroup's first K,V loads wait for this item only, not for a table read as well
  int32_t pad[5];
};
struct MergeItem {  // 16 bytes: a short turn that the decode kernel cut at the boundary of two shares
  int32_t s, t0, pslot0, n_chunks;  // pslot0: the decode kernel's slot (2 * workgroup + 0 / 1) of the first piece
};
// Header of the workspace (ints): counts written by the scheduler, a counter of the decode kernel, flags, and a 256-byte
// page of zeros (source of absent key rows).
constexpr int kHdrInts = 128;
constexpr int kHdrItems = 0, kHdrChunk = 1, kHdrSplitUnits = 2, kHdrPslots = 3, kHdrDecSessions = 4, kHdrDecTiles = 5,
              kHdrDecMerges = 6, kHdrFlags = kAttnHdrFlags;
static_assert(kHdrFlags < kAttnHdrInts && kAttnHdrInts <= 64, "the counts and flags lie in front of the zero page");
constexpr int kZeroPageInt = 64;
constexpr int kPartialFloats = 256 * 66;  // per workgroup: 64 accumulators + running max + running sum per thread
// A piece of a short turn (decode kernel): only the session's own rows, r = head * N + token (at most 32), packed:
// rows x 128 accumulators, then the rows' softmax references, then their sums.  Whole 128-byte lines are written and
// nothing else: a slot in the layout above would be 528 lines with 32 of their 128 bytes dirty, and writing such lines
// back cost the decode step 13 % of its time.
constexpr int kDecPartialFloats = 32 * 130;

struct SchedParams {
  const int32_t* cu_new_lens;
  const int32_t* prefix_lens;
  int32_t n_sessions, bmt, n_kv_heads, target, target_slots, c_min, coarse_ok;
  int32_t items_bound, merges_bound, pslots_bound;
  int32_t bmt_dec;      // sessions with at most this many new tokens go to the decode kernel (0: none do)
  int32_t* dec_s;       // their indices, in session order
  int32_t* dec_off;     // exclusive prefix sum of their key counts in 32-key tiles (one more entry: the total)
  int32_t* hdr;
  WorkItem* items;
  int32_t* merge_cnt;   // [merges_bound][n_kv_heads]: chunks of a split unit that have written their partial result
  const int32_t* table; // block table (may be null) and what is needed to find the ids of an item's first tiles
  int32_t table_stride, log_bs;
};

constexpr int kBN = 64;  // keys per tile
constexpr int kSchedThreads = 256;
constexpr int kSchedBuckets = 64;      // one per lane of a wave: the bucket offsets are a single wave-level scan
constexpr int kSchedMaxSessions = 4096;  // sessions whose lengths and unit offsets fit the scheduler's LDS tables

__device__ __forceinline__ int unit_tiles(int P, int N, int t0, int bmt) {
  return (P + min(N, t0 + bmt) + kBN - 1) / kBN;
}

// Inclusive scan over the 64 lanes of a wave with data-parallel moves: shifts by 1, 2, 4, 8 inside each row of 16
// lanes (a lane without a source adds 0), then the last lane of rows 0 and 2 added to rows 1 and 3, then lane 31 to
// rows 2 and 3.  (A shuffle per step goes through the LDS crossbar and takes ten times as long.)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_from(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, true);
}
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_from<0x111, 0xF>(v);  // row_shr:1
  v += dpp_from<0x112, 0xF>(v);  // row_shr:2
  v += dpp_from<0x114, 0xF>(v);  // row_shr:4
  v += dpp_from<0x118, 0xF>(v);  // row_shr:8
  v += dpp_from<0x142, 0xA>(v);  // row_bcast:15
  v += dpp_from<0x143, 0xC>(v);  // row_bcast:31
  return v;
}

// Maximum over the 64 lanes of a wave of values >= 0 (the same moves as the scan; a lane without a source sees 0);
// lane 63 holds the result.
__device__ __forceinline__ int wave_inclusive_max(int v) {
  v = max(v, dpp_from<0x111, 0xF>(v));
  v = max(v, dpp_from<0x112, 0xF>(v));
  v = max(v, dpp_from<0x114, 0xF>(v));
  v = max(v, dpp_from<0x118, 0xF>(v));
  v = max(v, dpp_from<0x142, 0xA>(v));
  v = max(v, dpp_from<0x143, 0xC>(v));
  return v;
}

// Inclusive scan of two ints per thread across the 256-thread block; the block totals come back through tot_a, tot_b.
__device__ __forceinline__ void block_inclusive_scan2(int& a, int& b, int (*wave_sums)[2], int& tot_a, int& tot_b) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  a = wave_inclusive_scan(a);
  b = wave_inclusive_scan(b);
  __syncthreads();
  if (lane == 63) {
    wave_sums[w][0] = a;
    wave_sums[w][1] = b;
  }
  __syncthreads();
  int base_a = 0, base_b = 0;
  for (int i = 0; i < w; ++i) {
    base_a += wave_sums[i][0];
    base_b += wave_sums[i][1];
  }
  tot_a = wave_sums[0][0] + wave_sums[1][0] + wave_sums[2][0] + wave_sums[3][0];
  tot_b = wave_sums[0][1] + wave_sums[1][1] + wave_sums[2][1] + wave_sums[3][1];
  a += base_a;
  b += base_b;
}

// One workgroup turns the ragged batch into the ordered work list.  All passes run over the flat list of units
// (session, query tile), one unit per thread per step, so a batch of one long session is as parallel as a batch of many
// short ones.  Which units are split, and which partial-result slots and counters their chunks get, follows from
// prefix sums in unit order: the same for every run, and a unit for whose chunks the workspace has no room is simply
// left whole (flag bit 0), never dropped.
__global__ __launch_bounds__(kSchedThreads) void attn_schedule_kernel(const SchedParams p) {
  __shared__ int unit_off[kSchedMaxSessions + 1];
  __shared__ int len_new[kSchedMaxSessions], len_prefix[kSchedMaxSessions], cu_of[kSchedMaxSessions];
  __shared__ int wave_sums[4][2];
  __shared__ unsigned long long total_tiles_s;
  __shared__ int max_nt_s, inv_min_nt_s;  // longest unit, and 0x7FFFFFFF - shortest unit (tiles; units with tiles only)
  __shared__ int hist[kSchedBuckets];
  __shared__ int n_items_s, n_split_s, n_pslot_s, chunk_s, flags_s;
  const int tid = threadIdx.x;
  const int S = p.n_sessions;
  if (tid >= kZeroPageInt && tid < kHdrInts) p.hdr[tid] = 0;
  for (int i = tid; i < p.merges_bound * p.n_kv_heads; i += kSchedThreads) p.merge_cnt[i] = 0;
  if (tid == 0) {
    total_tiles_s = 0ull;
    max_nt_s = 0;
    inv_min_nt_s = 0;
    n_items_s = 0;
    n_split_s = 0;
    n_pslot_s = 0;
    flags_s = 0;
  }
  if (tid < kSchedBuckets) hist[tid] = 0;
  // unit offsets: exclusive prefix sum of ceil(N_s / bmt); short turns: their count and their keys in 32-key tiles
  int U = 0, n_dec = 0, dec_total = 0;
  for (int base = 0; base < S; base += kSchedThreads) {
    const int s = base + tid;
    // the lengths are read from memory once and kept in LDS for the passes below
    const int cu_s = s < S ? p.cu_new_lens[s] : 0;
    const int N = s < S ? p.cu_new_lens[s + 1] - cu_s : 0;
    const int P = s < S ? p.prefix_lens[s] : 0;
    if (s < S) {
      len_new[s] = N;
      len_prefix[s] = P;
      cu_of[s] = cu_s;
    }
    int nq = N > 0 ? (N + p.bmt - 1) / p.bmt : 0, zero = 0, tot_q, tot_z;
    block_inclusive_scan2(nq, zero, wave_sums, tot_q, tot_z);
    if (s < S) unit_off[s] = U + nq - (N > 0 ? (N + p.bmt - 1) / p.bmt : 0);
    U += tot_q;
    if (p.bmt_dec > 0) {
      // Short turns (1 <= N_s <= bmt_dec) are not cut into work items: the decode kernel splits the concatenation of
      // their key ranges evenly among its workgroups, and needs their indices and the prefix sum of their lengths.
      const int is_dec = N >= 1 && N <= p.bmt_dec;
      const int nt = is_dec ? (P + N + 31) / 32 : 0;
      int ic = is_dec, itl = nt, tot_c, tot_t;
      block_inclusive_scan2(ic, itl, wave_sums, tot_c, tot_t);
      if (is_dec) {
        p.dec_s[n_dec + ic - 1] = s;
        p.dec_off[n_dec + ic - 1] = dec_total + itl - nt;
      }
      n_dec += tot_c;
      dec_total += tot_t;
    }
  }
  if (tid == 0) {
    unit_off[S] = U;
    if (p.bmt_dec > 0) p.dec_off[n_dec] = dec_total;
  }
  if (U == n_dec) {  // every unit is a short turn (each has exactly one), or there is none: nothing for the work list
    if (tid < 8) p.hdr[tid] = tid == kHdrDecSessions ? n_dec : (tid == kHdrDecTiles ? dec_total : 0);
    return;
  }
  __syncthreads();
  // unit u -> tiles it has to visit (0: none, it is past the list or a short turn), with its session and lengths
  struct Unit {
    int s, t0, P, N, nt;
  };
  auto unit = [&](int u) {
    Unit r{0, 0, 0, 0, 0};
    if (u >= U) return r;
    int lo = 0, hi = S;  // last s with unit_off[s] <= u
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (unit_off[mid] <= u)
        lo = mid;
      else
        hi = mid;
    }
    r.s = lo;
    r.t0 = (u - unit_off[lo]) * p.bmt;
    r.P = len_prefix[lo];
    r.N = len_new[lo];
    r.nt = r.N <= p.bmt_dec ? 0 : unit_tiles(r.P, r.N, r.t0, p.bmt);
    return r;
  };
  // A thread's units (u = tid, tid + 256, ...) and the way they are cut are worked out once and kept in registers
  // between the passes while there are at most kSchedCached of them per thread; longer lists recompute them.
  constexpr int kSchedCached = 4;
  const int n_rounds = (U + kSchedThreads - 1) / kSchedThreads;
  const bool cached = n_rounds <= kSchedCached;
  Unit uc[kSchedCached];
  // Block ids of a unit's first two key tiles: what its first (for most units: only) work item carries.  Their loads
  // start here and return while the passes below run.
  int ids0[kSchedCached][8];
  const bool has_table = p.table && p.table_stride > 0;
  auto first_ids_of = [&](int s, int first_tile, int (&ids)[8]) {
    const int32_t* table_row = p.table + (int64_t)s * p.table_stride;
#pragma unroll
    for (int i = 0; i < 8; ++i)  // (index clamped to the row: an entry past the session's keys is never used)
      ids[i] = has_table ? table_row[min((first_tile * kBN + 16 * i) >> p.log_bs, p.table_stride - 1)] : -1;
  };
  // pass 1: total number of (unit, key tile) pairs
  unsigned long long mine = 0;
  int longest = 0, inv_shortest = 0;
  auto note = [&](int nt) {
    mine += (unsigned long long)nt;
    if (nt > 0) {
      longest = max(longest, nt);
      inv_shortest = max(inv_shortest, 0x7FFFFFFF - nt);
    }
  };
  if (cached) {
#pragma unroll
    for (int r = 0; r < kSchedCached; ++r) {
      uc[r] = unit(r * kSchedThreads + tid);
      note(uc[r].nt);
      if (r < n_rounds && uc[r].nt > 0) first_ids_of(uc[r].s, 0, ids0[r]);
    }
  } else {
    for (int u = tid; u < U; u += kSchedThreads) note(unit(u).nt);
  }
  // (summed inside each wave first: atomics of all threads on the one LDS word run one after the other, and took
  // longer than every other step of this kernel)
  {
    // three scans of 20-bit pieces: none can overflow an int over 64 lanes (a thread's count is below 2^60)
    const int s0 = wave_inclusive_scan((int)(mine & 0xFFFFFull));
    const int s1 = wave_inclusive_scan((int)((mine >> 20) & 0xFFFFFull));
    const int s2 = wave_inclusive_scan((int)(mine >> 40));
    const unsigned long long wave_total =
        ((unsigned long long)(unsigned)s2 << 40) + ((unsigned long long)(unsigned)s1 << 20) + (unsigned)s0;
    longest = wave_inclusive_max(longest);
    inv_shortest = wave_inclusive_max(inv_shortest);
    if ((tid & 63) == 63 && wave_total) {
      atomicAdd(&total_tiles_s, wave_total);
      atomicMax(&max_nt_s, longest);
      atomicMax(&inv_min_nt_s, inv_shortest);
    }
  }
  __syncthreads();
  if (tid == 0) {
    // With at least two workgroup-sized units per slot, longest-first dispatch balances well without splitting
    // anything but the longest units; with fewer, every unit is cut so that there are about two pieces per slot.
    const long long wg_units = (long long)(U - n_dec) * p.n_kv_heads;
    const int target = (p.coarse_ok && wg_units >= 2ll * p.target_slots) ? p.target_slots : p.target;
    // C = ceil(total tiles * kv-heads / target): a single-precision estimate, then exact steps in integers
    const unsigned long long tot = total_tiles_s * (unsigned long long)p.n_kv_heads;
    long long c = (long long)((float)tot * (1.0f / (float)target));
    if (c > 0x3FFFFFFF) c = 0x3FFFFFFF;
    while (c < 0x3FFFFFFF && (unsigned long long)c * (unsigned long long)target < tot) ++c;
    while (c > 0 && (unsigned long long)(c - 1) * (unsigned long long)target >= tot) --c;
    // Units of (nearly) one length, and too few of them for the coarse rule: a single long session, or a batch of
    // equal ones.  Equal pieces are dispatched in whole rounds, so what counts is rounds x (piece + fixed cost), and
    // one round of longer pieces can beat two rounds of shorter ones.  Only cuts that are not finer than the one
    // above are tried (the workspace bounds are derived from it).
    const long long max_nt = max_nt_s, min_nt = 0x7FFFFFFF - inv_min_nt_s;
    if (target == p.target && max_nt > 0 && min_nt * 51 >= max_nt * 50 && c > 0) {
      constexpr long long kFixedTiles = 6;  // a work item's fixed cost (~11 us) in key tiles (~1.9 us)
      long long best_c = c, best_cost = 0x7FFFFFFFFFFFFFFFll;
      for (long long k = 1; k <= 64; ++k) {
        const long long ck = (max_nt + k - 1) / k;
        if (ck < c) break;
        const long long rounds = (wg_units * k + p.target_slots - 1) / p.target_slots;
        const long long cost = rounds * (ck + kFixedTiles);
        if (cost <= best_cost) {  // (of equal costs the finer cut: more pieces in flight)
          best_cost = cost;
          best_c = ck;
        }
      }
      c = best_c;
    }
    if (c < p.c_min) c = p.c_min;
    chunk_s = (int)c;
  }
  __syncthreads();
  const int C = chunk_s;
  // bucket of a chunk length: longer chunks get smaller bucket numbers (they are dispatched first).  Any monotone
  // function of the length will do, as long as both passes below use the same one.
  const float buckets_per_tile = (float)kSchedBuckets / (float)C;
  auto bucket_of = [&](int len) {
    const int b = (int)((float)(C - len) * buckets_per_tile);
    return b < 0 ? 0 : (b >= kSchedBuckets ? kSchedBuckets - 1 : b);
  };
  // How a unit is cut: chunks of `len` tiles, n_real of them, in slots pslot0 .. and with counter `merge` when it is
  // split (n_real > 1).  The running totals of chunks and of split units (carry_c, carry_m) go through the rounds in
  // unit order; a unit whose chunks would pass the end of the slots or of the counters stays whole, and so does every
  // split candidate after it.  (Every thread of the block calls this the same number of times: it holds barriers.)
  struct Cut {
    int len, n_real, pslot0, merge;
  };
  auto cut_of = [&](const Unit& un, int& carry_c, int& carry_m) {
    Cut c;
    const int nt = un.nt;
    const int nc = nt > 0 ? (nt + C - 1) / C : 0;
    c.len = nc > 0 ? (nt + nc - 1) / nc : 0;
    c.n_real = c.len > 0 ? (nt + c.len - 1) / c.len : 0;
    const bool want = c.n_real > 1;
    int ic = want ? c.n_real : 0, im = want ? 1 : 0, tot_c, tot_m;
    block_inclusive_scan2(ic, im, wave_sums, tot_c, tot_m);
    const bool fits = carry_c + ic <= p.pslots_bound && carry_m + im <= p.merges_bound;
    c.pslot0 = carry_c + ic - c.n_real;
    c.merge = carry_m + im - 1;
    if (want && !fits) {
      c.len = nt;
      c.n_real = 1;
      atomicOr(&flags_s, 1);
    }
    // slots and counters in use = the largest prefix sums that fitted (one LDS atomic per wave, not per unit: atomics
    // of many lanes on one word run one after the other)
    const int end_c = wave_inclusive_max(want && fits ? carry_c + ic : 0);
    const int end_m = wave_inclusive_max(want && fits ? carry_m + im : 0);
    if ((threadIdx.x & 63) == 63 && end_c) {
      atomicMax(&n_pslot_s, end_c);
      atomicMax(&n_split_s, end_m);
    }
    if (c.n_real <= 1) {
      c.pslot0 = -1;
      c.merge = -1;
    }
    carry_c += tot_c;
    carry_m += tot_m;
    return c;
  };
  // pass 2: histogram of chunk lengths
  auto count = [&](const Unit& un, const Cut& c) {
    if (c.n_real == 0) return;
    const int n_full = un.nt / c.len, rem = un.nt - n_full * c.len;  // n_full chunks of len tiles, one of rem
    if (n_full) atomicAdd(&hist[bucket_of(c.len)], n_full);
    if (rem) atomicAdd(&hist[bucket_of(rem)], 1);
  };
  Cut cc[kSchedCached];
  {
    int carry_c = 0, carry_m = 0;
    if (cached) {
#pragma unroll
      for (int r = 0; r < kSchedCached; ++r)
        if (r < n_rounds) {
          cc[r] = cut_of(uc[r], carry_c, carry_m);
          count(uc[r], cc[r]);
        }
    } else {
      for (int base = 0; base < U; base += kSchedThreads) {
        const Unit un = unit(base + tid);
        count(un, cut_of(un, carry_c, carry_m));
      }
    }
  }
  __syncthreads();
  if (tid < kSchedBuckets) {  // wave 0: exclusive prefix sum, hist[b] becomes the first list position of bucket b
    const int h = hist[tid];
    const int incl = wave_inclusive_scan(h);
    hist[tid] = incl - h;
    if (tid == kSchedBuckets - 1) n_items_s = incl;
  }
  __syncthreads();
  // pass 3: emit items
  auto emit = [&](const Unit& un, const Cut& c, const int (*ids_first)[8]) {  // ids_first: of chunk 0, or null
    if (c.n_real == 0) return;
    const int cu_s = cu_of[un.s];
    // four chunks at a time: their table reads are issued together, before the first item is written (one wait for
    // memory per group instead of one per chunk)
    for (int ch0 = 0; ch0 < c.n_real; ch0 += 4) {
      int ids[4][8];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int ch = ch0 + k;
        if (ch >= c.n_real) break;
        if (ch == 0 && ids_first) {
#pragma unroll
          for (int i = 0; i < 8; ++i) ids[k][i] = (*ids_first)[i];
        } else {
          first_ids_of(un.s, ch * c.len, ids[k]);
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int ch = ch0 + k;
        if (ch >= c.n_real) break;
        const int tb = ch * c.len, te = min(un.nt, tb + c.len);
        const int pos = atomicAdd(&hist[bucket_of(te - tb)], 1);
        if (pos < p.items_bound) {
          WorkItem w{un.s, un.t0, tb, te, c.n_real > 1 ? c.pslot0 + ch : -1, cu_s, un.N, un.P,
                     c.merge, c.pslot0, c.n_real, {-1, -1, -1, -1, -1, -1, -1, -1}, {0, 0, 0, 0, 0}};
#pragma unroll
          for (int i = 0; i < 8; ++i) w.first_ids[i] = ids[k][i];
          p.items[pos] = w;
        } else {
          atomicOr(&flags_s, 2);  // more units than total_new_tokens and n_sessions allow: the lengths on the device
                                  // disagree with the host's bounds, and this piece of work is not done
        }
      }
    }
  };
  if (cached) {
#pragma unroll
    for (int r = 0; r < kSchedCached; ++r)
      if (r < n_rounds) emit(uc[r], cc[r], &ids0[r]);
  } else {
    int carry_c = 0, carry_m = 0;
    for (int base = 0; base < U; base += kSchedThreads) {
      const Unit un = unit(base + tid);
      emit(un, cut_of(un, carry_c, carry_m), nullptr);
    }
  }
  __syncthreads();
  if (tid == 0) {
    p.hdr[kHdrItems] = min(n_items_s, p.items_bound);
    p.hdr[kHdrChunk] = C;
    p.hdr[kHdrSplitUnits] = n_split_s;
    p.hdr[kHdrPslots] = n_pslot_s;
    p.hdr[kHdrDecSessions] = n_dec;
    p.hdr[kHdrDecTiles] = dec_total;
    p.hdr[kHdrDecMerges] = 0;
    p.hdr[kHdrFlags] = flags_s;
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
  int32_t* hdr;
  const WorkItem* items;
  int32_t* merge_cnt;   // [split unit][kv-head]: chunks that have written their partial result
  float* partials;
  // attn_decode_kernel: the short turns' session indices and tile prefix sums (written by the scheduler), the first of
  // its partial-result slots, its list of sessions cut at the boundary of two shares and the room in that list
  const int32_t* dec_s;
  const int32_t* dec_off;
  MergeItem* dec_merges;
  int32_t dec_merges_bound;
  float* dec_partials;  // [2 * key ranges][n_kv_heads][dec_slot_floats], behind the work items' slots
  int32_t dec_slot_floats;  // room for the packed piece of the longest short turn the call admits (whole lines)
};


constexpr int kD = 128;  // head_dim
// A row sum above this (one probability of 2^40 or more, or an overflow) makes the softmax reference stale.
constexpr float kRefreshSum = 1.0995116e12f;  // 2^40

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

// The 32 output rows of a wave through a buffer of its own in LDS: every store instruction then writes whole 128-byte
// lines (the G heads of a token are neighbours in memory: a wave's rows, in (token, head) order, are 32 / G runs of
// G x 256 bytes), where the direct form writes 8 bytes per lane, i.e. sixteen separate pieces per line for the L2 to put
// together.  row_of_lane: this lane's row in (token, head) order; valid_bits: bit m set = row m is written.
constexpr int kOutRowBytes = 256 + 16;
__device__ __forceinline__ void store_out_rows_staged(char* stage, __bf16* first_row, int64_t token_stride_elems,
                                                      int rows_per_token, int row_of_lane, unsigned valid_bits,
                                                      const f32x16 (&acc)[4], float inv, int g2, int lane) {
  char* wr = stage + row_of_lane * kOutRowBytes + 8 * g2;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x4 v;
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = (__bf16)(acc[dt][4 * i + j] * inv);
      *reinterpret_cast<bf16x4*>(wr + 64 * dt + 16 * i) = v;
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int m = 4 * it + (lane >> 4);
    const int tok = m / rows_per_token, hd = m - tok * rows_per_token;
    if ((valid_bits >> m) & 1u) {
      const u32x4_t v = *reinterpret_cast<const u32x4_t*>(stage + m * kOutRowBytes + 16 * (lane & 15));
      *reinterpret_cast<u32x4_t*>(reinterpret_cast<char*>(first_row + tok * token_stride_elems + (int64_t)hd * kD) + 16 * (lane & 15)) = v;
    }
  }
}

// Lanes l and l^32 hold the two halves of one query's keys.  v_permlane32_swap_b32 a, b exchanges lanes 32..63 of a
// with lanes 0..31 of b, so starting from two copies of x it leaves a = low half twice, b = high half twice.
// Written as inline assembly: with this compiler the builtin hands back the first register for both results.
__device__ __forceinline__ void swap_halves(float x, float& lo_twice, float& hi_twice) {
  float a = x, b = x;
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));  // a pure function of a, b: free to be scheduled
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


typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// LDS tile layout shared by K and V (64 key rows x 256 bytes): rows are stored in groups of four; a group is the
// 1 KiB that one wave writes with one direct global->LDS load (lane l lands at group base + 16*l), groups are
// kGroupBytes apart (16 bytes of padding), and inside row r of a group the 16-byte chunk c sits at position
// c ^ ((r & 3) << 2).  With this, the 16 rows that a quarter-wave reads with ds_read_b128 (K fragments) and the
// 4 rows x 32 bytes that 16 lanes read with ds_read_b64_tr_b16 (V fragments) each cover all banks once.
constexpr int kGroupBytes = 1024 + 16;
constexpr int kTileBytes = 16 * kGroupBytes;  // 16640

#define SYMPH_GLDS16(src, dst)                                                                       \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),             \
                                   (__attribute__((address_space(3))) void*)(dst), 16, 0, 0)

// The same with the non-temporal cache policy (bit 1 of the last operand): for rows that are read once
#define SYMPH_GLDS16_NT(src, dst)                                                                    \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),             \
                                   (__attribute__((address_space(3))) void*)(dst), 16, 0, 2)

// One workgroup = one work item x one kv-head: 128 query rows (G heads x 128/G tokens) against the item's key tiles.
// Requires block_size >= 16 (a power of two): the 16 consecutive key rows of a staging group then lie in ONE block, so
// block ids are workgroup-uniform and a row address is scalar base + per-lane constant.
// LB = log2(block_size) when it is 4 (the common 16-token block), else 0 = runtime.
//
// Pipeline, iteration j (tiles are double-buffered in LDS, buffers are separate arrays so that the compiler can tell
// which loads an LDS read has to wait for):
//   start : direct global->LDS loads of K(j+2) and V(j+1) are issued (no registers, no LDS store instructions);
//   block : S(j+1) = K(j+1) Q^T on the matrix cores  ||  online softmax of S(j) on the vector ALU  -> P(j);
//   then  : O += V(j)^T P(j);   end: wait for the loads, one barrier.
// The first product of the NEXT tile is independent of the softmax of the current one, so one wave keeps the matrix
// pipe and the vector ALU busy at the same time instead of alternating between them.
template <int G, int LB>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(const MfmaParams p) {
  constexpr int BMT = 128 / G;  // query tokens per tile
  __shared__ __attribute__((aligned(16))) char K0[kTileBytes];
  __shared__ __attribute__((aligned(16))) char K1[kTileBytes];
  __shared__ __attribute__((aligned(16))) char V0[kTileBytes];
  __shared__ __attribute__((aligned(16))) char V1[kTileBytes];

  const int Hkv = p.n_kv_heads;
  const int item_idx = blockIdx.x / Hkv;
  __shared__ int merges_here;  // set for the chunk of a split unit that arrives last
  // The array covers the whole grid, so the item is read beside the count, not after it: one trip to memory less in
  // front of the first K,V loads.  (The empty statement makes the compiler issue both loads before the branch.)
  const WorkItem it = p.items[item_idx];
  const int n_items = p.hdr[kHdrItems];
  asm volatile("" ::"s"(it.s), "s"(it.pslot), "s"(it.n_chunks), "s"(it.first_ids[0]), "s"(it.first_ids[7]), "s"(n_items));
  if (item_idx >= n_items) return;
  const int kvh = blockIdx.x - item_idx * Hkv;
  const int s = it.s;
  const int t0 = it.t0;
  const int cu_s = it.cu_s;
  const int N = it.n_new;
  const int P = it.n_prefix;
  const int lb = LB ? LB : p.log_bs;
  const int bs_mask = (1 << lb) - 1;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int n = lane & 31;  // query column of this lane inside the wave's 32 rows; also its A-operand row
  const int g2 = lane >> 5;

  // Query row of this lane.  The tile's 128 / G tokens are dealt to the waves in order, 32 / G tokens x G heads each
  // (head-major inside the wave), so that the tokens a tile does not have (a session's last tile, a short turn) leave
  // WHOLE waves without rows.  Such a wave only issues its share of the K,V loads and keeps the barriers: it skips the
  // matrix and vector work, which would be padding, and leaves those pipes to the workgroup that shares the CU (a
  // one-token turn fills 4 of the 128 rows: all in wave 0).
  constexpr int TW = BMT / 4;  // tokens per wave
  const int hh = n / TW;
  const int tt = wave * TW + (n - hh * TW);
  const bool q_valid = t0 + tt < N;
  const bool wave_works = t0 + wave * TW < N;
  const int tok = t0 + tt;
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
  // tiles below fast_end lie entirely inside the paged prefix: every row comes from the pool
  const int fast_end = min(tile_end, P / kBN);

  // ---- global -> LDS: wave w writes row group 4*i + w (rows 16*i + 4*w .. +3 of the tile) with its i-th load;
  // lane l covers row 4*w + l/16 of the 16-row group and holds logical chunk (l % 16) ^ ((l/16) << 2) of it.
  const bool has_table = p.table != nullptr && p.table_stride > 0;
  const int32_t* table_row = p.table + (int64_t)s * p.table_stride;
  const int dma_row = 4 * wave + (lane >> 4);                          // row inside a 16-row group
  const int dma_chunk = (lane & 15) ^ (((lane >> 4) & 3) << 2);        // logical 16-byte chunk this lane fetches
  const unsigned row_bytes = p.row_bytes;
  const unsigned voff = (unsigned)dma_row * row_bytes + (unsigned)kvh * 256u + (unsigned)dma_chunk * 16u;
  const char* k_bytes = reinterpret_cast<const char*>(p.k_layer);
  const char* v_bytes = reinterpret_cast<const char*>(p.v_layer);

  // Block ids of the tile's four 16-row groups.  The table entries are fetched (vector loads, every lane the same
  // address) a whole iteration before they are needed and only then moved to scalar registers: asking for the value
  // right after issuing the load would also wait for the K,V loads issued just before it.
  int ids[4];   // scalar: ids of the tile whose K rows are loaded next
  int ids_raw;  // in flight: lane i < 4 holds the id of group i of the tile after that
  auto fetch_ids = [&](int tile) {
    const int jb = (tile * kBN + 16 * (lane & 3)) >> lb;
    ids_raw = has_table ? table_row[min(jb, p.table_stride - 1)] : -1;
  };
  auto take_ids = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) ids[i] = __builtin_amdgcn_readlane(ids_raw, i);
  };
  // Issue the loads of one tile of K or of V into an LDS buffer.  Rows that do not exist (past the session's keys, or
  // named by a block id outside the cache) are read from the page of zeros, so they are finite and add nothing.
  auto issue_tile = [&](const char* pool_bytes, const __bf16* new_rows, char* lds_buf, int tile) {
    // one comparison of the largest id (as unsigned: a negative id is huge)
    const unsigned id_max = max(max((unsigned)ids[0], (unsigned)ids[1]), max((unsigned)ids[2], (unsigned)ids[3]));
    const bool fast = tile < fast_end && id_max < (unsigned)p.n_blocks;
    if (__builtin_expect(fast, 1)) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint64_t off = (uint64_t)(unsigned)ids[i] * p.block_bytes;
        if (LB != 4) off += (uint64_t)((tile * kBN + 16 * i) & bs_mask) * row_bytes;
        // Scalar base + 32-bit lane offset, kept apart for the compiler: with 64-bit per-lane addresses the issue of
        // such a load waits for the matrix instructions of the SIMD's other wave (microbenchmark: eight loads take
        // 290 clocks in this form whatever the other wave does, and 500-2100 in the other while it runs MFMAs).
        const char* base = pool_bytes + off;
        unsigned lane_off = voff;
        asm("" : "+s"(base), "+v"(lane_off));
        SYMPH_GLDS16(base + lane_off, lds_buf + (4 * i + wave) * kGroupBytes);
      }
      asm volatile("; end of the scalar-base loads");  // keeps the last one from being merged with the other path's
    } else {
      // rare path: its per-lane address pieces are derived here, from a lane id the optimiser cannot see through, so
      // that they do not occupy registers throughout the main loop
      int l = lane;
      asm volatile("" : "+v"(l));
      const int row = 4 * wave + (l >> 4);
      const unsigned in_row = (unsigned)kvh * 256u + (unsigned)((l & 15) ^ (((l >> 4) & 3) << 2)) * 16u;
      const char* const zeros = reinterpret_cast<const char*>(p.hdr + kZeroPageInt) + (l & 15) * 16;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = tile * kBN + 16 * i + row;
        const unsigned b = (unsigned)ids[i];
        const bool in_pool = key < P && (key >> lb) < p.table_stride && b < (unsigned)p.n_blocks;
        const bool in_new = key >= P && key < total_keys;
        const char* src = zeros;
        if (in_pool)
          src = pool_bytes + (uint64_t)b * p.block_bytes + (uint64_t)(key & bs_mask) * row_bytes + in_row;
        else if (in_new)
          src = reinterpret_cast<const char*>(new_rows) + (uint64_t)(cu_s + key - P) * row_bytes + in_row;
        SYMPH_GLDS16(src, lds_buf + (4 * i + wave) * kGroupBytes);
      }
    }
  };

  // ---- LDS reads.  K fragment (A operand of S^T = K Q^T): lane (n, g2) reads 16 bytes of key row
  // key_of_row(n) (+32 for the second block), logical chunk 2*st + g2.
  const int krow = key_of_row(n);
  const int k_lane = (krow >> 2) * kGroupBytes + (krow & 3) * 256 + g2 * 16;
  int k_off[4];  // byte offset for st >> 1 == q: chunk pair position q ^ (row & 3)
#pragma unroll
  for (int q = 0; q < 4; ++q) k_off[q] = k_lane + 64 * (q ^ (krow & 3));
  // V fragment (A operand of O^T += V^T P^T) via the transposing read: 16 lanes read 4 rows x 32 bytes and each gets
  // one column (4 consecutive keys of one d).  Lane group lane/16 = 2*g2 + dhalf, i16 = lane % 16:
  // row = 8*g2 + i16/4 (+ 32*kb + 16*u + 4*half), bytes 64*dt + 32*dhalf + 8*(i16 % 4) of the row.
  const int i16 = lane & 15;
  const int vrow = 8 * g2 + (i16 >> 2);
  const int v_lane = (vrow >> 2) * kGroupBytes + (vrow & 3) * 256 + 32 * ((lane >> 4) & 1) + 8 * (i16 & 3);
  int v_off[4];  // byte offset for d tile dt: chunk quad position dt ^ (row & 3)
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) v_off[dt] = v_lane + 64 * (dt ^ (vrow & 3));

  f32x16 o_acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o_acc[dt][e] = 0.f;
  float m_run = -INFINITY;  // running max of raw scores (before scale)
  float l_run = 0.f;        // this lane's share of the running sum
  const float cs = p.scale_log2e;
  const int q_limit = P + tok;  // last key this query may see
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  // S^T of one tile (64 keys x 32 queries per wave) on the matrix cores
  auto qk = [&](const char* kbuf, f32x16 (&sc)[2]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) sc[kb][e] = 0.f;
    {
      // the two 32-key blocks alternate, so consecutive MFMAs never wait for each other's accumulator
#pragma unroll
      for (int st = 0; st < 8; ++st)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(kbuf + k_off[st >> 1] + 32 * (st & 1) + kb * 8 * kGroupBytes);
          sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[st], sc[kb], 0, 0, 0);
        }
    }
  };
  // causal mask: only tiles that reach past the first query's limit
  auto mask = [&](f32x16 (&sc)[2], int tile) {
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
  };
  // Online softmax on the vector ALU, one query per lane (lanes l and l^32 split its keys), with a STALE reference:
  // probabilities are 2^((s - m_ref) * scale') for a reference m_ref that is NOT the running maximum but the maximum
  // at the time it was last refreshed.  Numerator and denominator carry the same factor, so the result is the exact
  // softmax as long as nothing overflows, and bf16 / fp32 keep their relative precision at any magnitude.  The
  // reference is refreshed (below) only when a tile's row sum shows that some score exceeds it by more than
  // kRefreshLog2, which after the first tile practically never happens; the per-tile maximum, the rescale factor
  // and the rescaling of the accumulators thereby leave the loop.
  // reference := max(reference, maximum of this tile), in log2 units; returns the factor by which everything
  // accumulated so far has to be rescaled (0 for a first reference, 1 where nothing moved)
  auto raise_reference = [&](const f32x16 (&sc)[2], float& mb) {
    float mx = sc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[kb][e]);
    mx = max_across_halves(mx);
    const float m_new = fmaxf(m_run, mx * cs);
    // a row that has seen no key yet (a work item may start past its causal limit) keeps m_run = -inf, which the
    // merge step reads as "no contribution"; its exponent arguments use 0 so that they stay finite
    const float a = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    mb = (m_new == -INFINITY) ? 0.f : m_new;
    return a;
  };
  // ... then the bf16 probabilities, one 32-key half at a time: the first half follows the statistics directly (in
  // the block that is otherwise almost pure matrix work), the second half runs beside the next tile's first product,
  // so that both blocks of the pipeline carry a similar mix of matrix and vector work whatever block the other
  // workgroup of the CU happens to be in
  auto softmax_exp_half = [&](const f32x16& sc, float mb, bf16x8 (&pb)[2]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      pb[e >> 3][e & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sc[e], cs, -mb));
    }
  };
  // row sum of the ROUNDED probabilities (the values the second product uses), two per instruction
  auto row_sum = [&](const bf16x8 (&pb)[2][2]) {
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
    return ps0 + ps1;
  };
  // Refresh of a stale reference (rare): rescale what has been accumulated, redo this tile's probabilities.
  auto refresh_reference = [&](const f32x16 (&sc)[2], float& mb, bf16x8 (&pb)[2][2], float& ps) {
    const float a = raise_reference(sc, mb);
    l_run *= a;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o_acc[dt][e] *= a;
    softmax_exp_half(sc[0], mb, pb[0]);
    softmax_exp_half(sc[1], mb, pb[1]);
    ps = row_sum(pb);
  };
  auto wait_loads_and_sync = [&]() {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's global->LDS loads have landed
    __syncthreads();
  };

  // Pipeline.  K(t) lives in K[t' & 1], V(t) in V[t' & 1] with t' = t - tile_begin.  Iteration j issues the loads
  // of K(j+2) and V(j+1) and then runs two straight-line blocks in which the matrix pipe and the vector ALU work on
  // INDEPENDENT data, so that one wave keeps both busy:
  //   block A:  S(j+1) = K(j+1) Q^T   (matrix)   ||   exponentials of S(j) -> P(j), row sums     (vector)
  //   block B:  O += V(j)^T P(j)      (matrix)   ||   running max / rescale factor of S(j+1)      (vector)
  // A wave issues in order, so the instruction stream itself has to alternate between the two kinds; the
  // sched_group_barrier sequences ask the scheduler for that interleaving and for LDS reads that run several matrix
  // instructions ahead of their use (a read issued right before its MFMA exposes the full LDS latency every time).
  f32x16 s_even[2], s_odd[2];  // scores of the even and of the odd tiles (counted from tile_begin)
  int ids_v[4];  // ids of the tile whose V rows are loaded next
  {
    // the ids of the first two tiles came with the work item
#pragma unroll
    for (int i = 0; i < 4; ++i) ids[i] = it.first_ids[i];
    issue_tile(k_bytes, p.k_new, K0, tile_begin);
    issue_tile(v_bytes, p.v_new, V0, tile_begin);
    if (tile_begin + 1 < tile_end) {
#pragma unroll
      for (int i = 0; i < 4; ++i) ids[i] = it.first_ids[4 + i];
      issue_tile(k_bytes, p.k_new, K1, tile_begin + 1);
    }
  }
  // The first product needs K0 only: V0 and K1, issued after it, may still be on their way (loads return in order).
  if (tile_begin + 1 < tile_end)
    __builtin_amdgcn_s_waitcnt(0x0F70 | 8);  // vmcnt(8)
  else
    __builtin_amdgcn_s_waitcnt(0x0F70 | 4);  // vmcnt(4)
  __syncthreads();
  if (wave_works) qk(K0, s_even);
#pragma unroll
  for (int i = 0; i < 4; ++i) ids_v[i] = ids[i];  // ids of tile b+1
  fetch_ids(tile_begin + 2);                      // taken at the top of the first iteration
  float mb_cur = 0.f;  // reference of the exponentials, in log2 units
  bf16x8 pb[2][2];     // P(j); its first half is produced one block ahead of the second
  if (wave_works) {
    mask(s_even, tile_begin);
    raise_reference(s_even, mb_cur);   // first reference: the maximum of the first tile
    softmax_exp_half(s_even[0], mb_cur, pb[0]);
  }
  // Every wave has read all of K0 for the first product before any wave overwrites it (the first iteration loads
  // K(tile_begin + 2) into K0), and V0 and K1 have landed for all waves.  Later iterations end with the same pair.
  wait_loads_and_sync();

  auto iteration = [&](const int j, auto par_c) {
    constexpr int PAR = decltype(par_c)::value;
    char* const k_same = PAR ? K1 : K0;   // held K(j), free now: receives K(j+2)
    char* const k_other = PAR ? K0 : K1;  // holds K(j+1)
    char* const v_same = PAR ? V1 : V0;   // holds V(j)
    char* const v_other = PAR ? V0 : V1;  // held V(j-1), free now: receives V(j+1)
    f32x16 (&s_cur)[2] = PAR ? s_odd : s_even;   // S(j)
    f32x16 (&s_nxt)[2] = PAR ? s_even : s_odd;   // receives S(j+1)
    if (j + 1 < tile_end) {
      int keep[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { keep[i] = ids[i]; ids[i] = ids_v[i]; }
      issue_tile(v_bytes, p.v_new, v_other, j + 1);   // ids of tile j+1
#pragma unroll
      for (int i = 0; i < 4; ++i) ids[i] = keep[i];
    }
    if (j + 2 < tile_end) issue_tile(k_bytes, p.k_new, k_same, j + 2);
    if (wave_works) {
    // ---- block A
    qk(k_other, s_nxt);                          // S(j+1)   (garbage, and discarded below, when j+1 == tile_end)
    softmax_exp_half(s_cur[1], mb_cur, pb[1]);   // second half of P(j)
    float ps = row_sum(pb);
    __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);      // K fragments: six reads up front
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // one MFMA of S(j+1)
      if (g < 10) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);    // vector ALU: scale, convert, sum
      __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);    // one exponential
    }
    // keep the probabilities (and with them the exponentials) in this block: without a use here the compiler sinks
    // them past the branch below, next to the second product
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int u = 0; u < 2; ++u) asm volatile("" : "+v"(pb[kb][u]));
    asm volatile("" : "+v"(ps));
    // The reference is stale when some score exceeds it by more than 40 in log2 units (then the row sum is huge,
    // infinite or NaN), or when a row that had seen no key now has one.  Rare: redo this tile's probabilities from
    // its scores, which are still in registers, against a refreshed reference.
    if (__any(!(ps <= kRefreshSum) || (m_run == -INFINITY && ps > 0.f))) refresh_reference(s_cur, mb_cur, pb, ps);
    l_run += ps;
    mask(s_nxt, j + 1);
    // ---- block B
    // O += V(j)^T P(j)  ||  first half of P(j+1), in an explicit order: each of the 16 slots holds the two LDS reads
    // of the MFMA four slots ahead, one MFMA, and the scale / exponential (/ convert) of one score; nothing moves
    // between slots.
    bf16x8 pb_first[2];
    {
      auto v_frag = [&](int g) {  // operand of MFMA g = ((kb * 2 + u) * 4 + dt)
        const char* vp = v_same + v_off[g & 3] + (8 * (g >> 3) + 4 * ((g >> 2) & 1)) * kGroupBytes;
        const s16x4 lo = lds_read_tr16(reinterpret_cast<const __bf16*>(vp));
        const s16x4 hi = lds_read_tr16(reinterpret_cast<const __bf16*>(vp + kGroupBytes));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      };
      bf16x8 frag[16];
      float pe[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) frag[g] = v_frag(g);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < 16; ++g) {
        if (g + 4 < 16) frag[g + 4] = v_frag(g + 4);
        o_acc[g & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[g], pb[g >> 3][(g >> 2) & 1], o_acc[g & 3], 0, 0, 0);
        pe[g] = __builtin_amdgcn_exp2f(fmaf(s_nxt[0][g], cs, -mb_cur));
        asm volatile("" : "+v"(pe[g]));  // evaluated in this slot (a value without side effects is otherwise placed
                                         // next to its use, after the last slot)
        if (g & 1) {
          pb_first[g >> 3][(g & 7) - 1] = (__bf16)pe[g - 1];
          pb_first[g >> 3][g & 7] = (__bf16)pe[g];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    pb[0][0] = pb_first[0];   // (garbage, and never used, when there was no tile j+1)
    pb[0][1] = pb_first[1];
    asm volatile("" : "+v"(pb[0][0]), "+v"(pb[0][1]));   // computed here, not after the barrier
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) ids_v[i] = ids[i];      // the next V tile is j+2
    wait_loads_and_sync();
  };
  // Before each iteration the ids fetched an iteration ago become scalar and the fetch of the next ones starts (it
  // completes under the wait at the end of the iteration).
  auto step = [&](int j, auto par_c) {
    take_ids();         // ids of tile j+2
    fetch_ids(j + 3);   // index clamped to the table: harmless past the last tile
    iteration(j, par_c);
  };
  for (int j = tile_begin; j < tile_end; j += 2) {
    step(j, std::integral_constant<int, 0>{});
    if (j + 1 < tile_end) step(j + 1, std::integral_constant<int, 1>{});
  }

  // rows of this wave in (token, head) order, and which of them exist
  const int row_m = (n - hh * TW) * G + hh;
  const int n_tok_here = min(max(N - (t0 + wave * TW), 0), TW);           // tokens of this wave's TW that exist
  const unsigned valid_bits = n_tok_here * G >= 32 ? 0xFFFFFFFFu : ((1u << (n_tok_here * G)) - 1u);
  char* const out_stage = wave == 0 ? K0 : (wave == 1 ? K1 : (wave == 2 ? V0 : V1));
  __bf16* const out_first = p.out + ((int64_t)(cu_s + t0 + wave * TW) * p.n_q_heads + kvh * G) * kD;
  if (it.pslot < 0) {
    const float l_tot = sum_across_halves(l_run);
    if (wave_works)   // (every wave is past the last barrier of the loop: the tile buffers are free)
      store_out_rows_staged(out_stage, out_first, (int64_t)p.n_q_heads * kD, G, row_m, valid_bits, o_acc, 1.0f / l_tot, g2,
                            lane);
  } else {
    // Register dump, one float per thread per store: fully coalesced.  The chunks of a unit may run on different XCDs,
    // whose L2 caches do not see each other's lines, so everything that passes between them is written and read at
    // device scope (each access goes to the point where the XCDs agree) instead of flushing and invalidating whole
    // caches around the hand-over: a release / acquire fence pair at device scope per chunk cost a quarter of the
    // kernel's time on a batch that is all split units.
    float* part = p.partials + ((int64_t)it.pslot * Hkv + kvh) * kPartialFloats + tid;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e)
        __hip_atomic_store(part + (dt * 16 + e) * 256, o_acc[dt][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(part + 64 * 256, m_run, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(part + 65 * 256, l_run, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // The chunk that arrives last combines all of them (no further kernel).  Every wave waits until its stores have
    // been performed, then one thread counts the chunk in.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    if (tid == 0)
      merges_here = __hip_atomic_fetch_add(p.merge_cnt + (int64_t)it.merge * Hkv + kvh, 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT) == it.n_chunks - 1;
    __syncthreads();
    if (!merges_here) return;
    // out = sum_c w_c O_c / sum_c w_c l_c with w_c = 2^(m_c - max_c m_c), m_c being chunk c's softmax reference in log2
    // units (-inf: the chunk saw no key of the row).  All chunks are read back in chunk order, this one's too, so the
    // result does not depend on which chunk came last.  Same thread -> (row, d) mapping as the dump above.
    const float* first = p.partials + ((int64_t)it.pslot0 * Hkv + kvh) * kPartialFloats + tid;
    const int64_t chunk_stride = (int64_t)Hkv * kPartialFloats;
    float M = -INFINITY;
    auto peer = [](const float* q) {  // a value another workgroup wrote during this launch
      return __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    for (int ch = 0; ch < it.n_chunks; ++ch) M = fmaxf(M, peer(first + ch * chunk_stride + 64 * 256));
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o_acc[dt][e] = 0.f;
    float L = 0.f;
    for (int ch = 0; ch < it.n_chunks; ++ch) {
      const float* src = first + ch * chunk_stride;
      const float mc = peer(src + 64 * 256);
      const float w = (mc == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mc - M);
      L += w * peer(src + 65 * 256);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[dt][e] = fmaf(w, peer(src + (dt * 16 + e) * 256), o_acc[dt][e]);
    }
    const float l_tot = sum_across_halves(L);
    if (wave_works)
      store_out_rows_staged(out_stage, out_first, (int64_t)p.n_q_heads * kD, G, row_m, valid_bits, o_acc, 1.0f / l_tot, g2,
                            lane);
  }
}

// ------------------------------------------------------------------------------------------------------------
// Short turns (decode-like rows): a session whose new rows fit one wave (n_new * G <= 32) reads its whole K,V for
// 32 query rows or fewer, so the work is moving K,V, not arithmetic.  The short turns' key ranges, laid end to end,
// are cut into equal ranges; a workgroup takes one range for a group of kv-heads, ONE WAVE PER KV-HEAD (eight waves
// for the usual eight heads, else single-wave workgroups).  A wave loads each 32-key tile of its head into an LDS
// buffer of its own (direct global->LDS loads) and uses it; the waves of a workgroup therefore read the eight 256-byte
// slices of the same 2 KiB token rows at the same time, kept together by a barrier per tile, and DRAM sees whole rows
// (a microbenchmark of this load stream: 7.0 TB/s as full rows, 6.7 as independent streams of slices, each pinned to
// an XCD, which is what one workgroup per kv-head gave).  A wave only alternates between "load a tile" and "use it",
// and using it is short, so what keeps HBM busy is the number of waves waiting for a tile: eight per CU, eight tiles
// (133 KiB) on their way nearly all the time.  (Double buffers per wave would halve the waves that fit, and a wave
// cannot keep a second, slower load in the background: loads return in order.)  Same fragment layouts, same
// transposed scores and same stale-reference softmax as attn_mfma_kernel; a wave owns all keys of its range, so its
// result needs no combining inside the workgroup.
// ------------------------------------------------------------------------------------------------------------
constexpr int kSub = 32;                    // keys per tile of this kernel
constexpr int kSubBytes = 8 * kGroupBytes;  // 8320
constexpr int kDecWaveBytes = 2 * kSubBytes;  // K and V of one tile, per wave

template <int G, int LB, int HW>
__global__ __launch_bounds__(64 * HW, HW == 8 ? 1 : 2) void attn_decode_kernel(const MfmaParams p) {
  constexpr int BMTD = 32 / G;   // query tokens this kernel covers per session
  static_assert(kDecPartialFloats * 4 <= kDecWaveBytes, "a wave stages its piece in its own tile buffers");
  __shared__ __attribute__((aligned(16))) char lds[HW * kDecWaveBytes];

  // Even split: the short turns' key ranges, laid end to end, are cut into equal ranges of 32-key tiles, whatever the
  // sessions' lengths.  A range covers the end of one session, whole sessions and the start of another: one segment
  // each, processed one after the other.  A session that lies in one range is finished here; the pieces of one that
  // spans several ranges go to the merge kernel.
  const int Hkv = p.n_kv_heads;
  const int n_groups = Hkv / HW;                 // groups of HW kv-heads: one wave per head of the group
  const int wg = blockIdx.x / n_groups;          // the range
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kvh = (blockIdx.x - wg * n_groups) * HW + wave;
  const int n_dec = p.hdr[kHdrDecSessions];
  const int total = p.hdr[kHdrDecTiles];
  const int n_ranges = (int)gridDim.x / n_groups;
  const int per_wg = (total + n_ranges - 1) / n_ranges;
  const int range_begin = wg * per_wg;
  const int range_end = min(total, range_begin + per_wg);
  if (range_begin >= range_end) return;
  const int lb = LB ? LB : p.log_bs;
  const int bs_mask = (1 << lb) - 1;
  int unit;  // last one that starts at or before range_begin
  {
    int lo = 0, hi = n_dec;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.dec_off[mid] <= range_begin)
        lo = mid;
      else
        hi = mid;
    }
    unit = lo;
  }
  for (int pos = range_begin; pos < range_end; ++unit) {
  const int unit_begin = p.dec_off[unit], unit_end = p.dec_off[unit + 1];
  const int s = p.dec_s[unit];
  const int cu_s = p.cu_new_lens[s];
  const int N = p.cu_new_lens[s + 1] - cu_s;
  const int P = p.prefix_lens[s];
  const int u_begin = pos - unit_begin;                        // this segment: tiles [u_begin, u_end) of the session
  const int u_end = min(range_end, unit_end) - unit_begin;
  const bool whole = u_begin == 0 && u_end == unit_end - unit_begin;
  const bool at_range_start = pos == range_begin;
  pos = unit_begin + u_end;

  const int lane = tid & 63;
  const int n = lane & 31;
  const int g2 = lane >> 5;
  // a wave holds the 32 query rows of its kv-head: row n = head n / BMTD, token n % BMTD
  const int hh = n / BMTD;
  const int tt = n - hh * BMTD;
  const bool q_valid = tt < N;
  const int head = kvh * G + hh;

  bf16x8 qreg[8];
  {
    const __bf16* qp = p.q + ((int64_t)(cu_s + (q_valid ? tt : 0)) * p.n_q_heads + head) * kD + 8 * g2;
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
  const int fast_end = min(u_end, P / kSub);  // tiles below lie entirely inside the paged prefix

  const bool has_table = p.table != nullptr && p.table_stride > 0;
  const int32_t* table_row = p.table + (int64_t)s * p.table_stride;
  const unsigned row_bytes = p.row_bytes;
  // a wave loads all eight row groups of a tile: lane l fetches row l/16 of the group's four, logical 16-byte chunk
  // (l % 16) ^ ((l/16) << 2)
  const unsigned voff = (unsigned)(lane >> 4) * row_bytes + (unsigned)kvh * 256u +
                        (unsigned)((lane & 15) ^ (((lane >> 4) & 3) << 2)) * 16u;
  const char* k_bytes = reinterpret_cast<const char*>(p.k_layer);
  const char* v_bytes = reinterpret_cast<const char*>(p.v_layer);
  char* const my_lds = lds + wave * kDecWaveBytes;  // K, then V

  // Ids of the two 16-row blocks of tile u (index clamped to the table); uniform addresses in read-only memory, so
  // these are scalar loads that do not count among the vector loads the waits below wait for.
  struct Ids {
    int a, b;
  };
  auto fetch_ids = [&](int u) {
    typedef const int32_t __attribute__((address_space(4))) * ConstTable;
    ConstTable row = (ConstTable)(uintptr_t)table_row;
    Ids r{-1, -1};
    if (has_table) {
      r.a = row[min((u * kSub) >> lb, p.table_stride - 1)];
      r.b = row[min((u * kSub + 16) >> lb, p.table_stride - 1)];
    }
    return r;
  };
  // The K rows (which = 0) or the V rows (1) of tile u into this wave's buffer for them: eight loads
  auto issue_half = [&](const int which, int u, const Ids ids) {
    char* const buf = my_lds + which * kSubBytes;
    const char* const pool = which ? v_bytes : k_bytes;
    const bool fast = u < fast_end && max((unsigned)ids.a, (unsigned)ids.b) < (unsigned)p.n_blocks;
    if (fast) {
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        uint64_t off = (uint64_t)(unsigned)(g < 4 ? ids.a : ids.b) * p.block_bytes + (uint64_t)(4 * (g & 3)) * row_bytes;
        if (LB != 4) off += (uint64_t)((u * kSub + 16 * (g >> 2)) & bs_mask) * row_bytes;
        const char* base = pool + off;  // scalar base + 32-bit lane offset, as in attn_mfma_kernel
        unsigned lane_off = voff;
        asm("" : "+s"(base), "+v"(lane_off));
        SYMPH_GLDS16_NT(base + lane_off, buf + g * kGroupBytes);  // every cached row is read once per kv-head
      }
      asm volatile("; end of the scalar-base loads");
    } else {
      const unsigned in_row = (unsigned)kvh * 256u + (unsigned)((lane & 15) ^ (((lane >> 4) & 3) << 2)) * 16u;
      const char* const zeros = reinterpret_cast<const char*>(p.hdr + kZeroPageInt) + (lane & 15) * 16;
      const char* const fresh = reinterpret_cast<const char*>(which ? p.v_new : p.k_new);
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        const int key = u * kSub + 4 * g + (lane >> 4);
        const unsigned bid = (unsigned)(g < 4 ? ids.a : ids.b);
        const bool in_pool = key < P && (key >> lb) < p.table_stride && bid < (unsigned)p.n_blocks;
        const bool in_new = key >= P && key < total_keys;
        const char* src = zeros;
        if (in_pool)
          src = pool + (uint64_t)bid * p.block_bytes + (uint64_t)(key & bs_mask) * row_bytes + in_row;
        else if (in_new)
          src = fresh + (uint64_t)(cu_s + key - P) * row_bytes + in_row;
        SYMPH_GLDS16(src, buf + g * kGroupBytes);
      }
    }
  };

  // ---- LDS reads: the fragment layouts of attn_mfma_kernel, for one 32-key block
  const int krow = key_of_row(n);
  const int k_lane = (krow >> 2) * kGroupBytes + (krow & 3) * 256 + g2 * 16;
  int k_off[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) k_off[q] = k_lane + 64 * (q ^ (krow & 3));
  const int i16 = lane & 15;
  const int vrow = 8 * g2 + (i16 >> 2);
  const int v_lane = (vrow >> 2) * kGroupBytes + (vrow & 3) * 256 + 32 * ((lane >> 4) & 1) + 8 * (i16 & 3);
  int v_off[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) v_off[dt] = v_lane + 64 * (dt ^ (vrow & 3));

  f32x16 o_acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o_acc[dt][e] = 0.f;
  float m_run = -INFINITY;  // softmax reference in log2 units, -inf: no key seen yet
  float mb = 0.f;           // the same, finite
  float l_run = 0.f;
  const float cs = p.scale_log2e;
  const int q_limit = P + tt;
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  auto exps = [&](const f32x16& sc, bf16x8 (&pb)[2]) {
#pragma unroll
    for (int e = 0; e < 16; ++e) pb[e >> 3][e & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sc[e], cs, -mb));
    float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8 v = pb[u];
      ps0 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[0], v[1]}, ones, ps0, false);
      ps1 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[2], v[3]}, ones, ps1, false);
      ps0 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[4], v[5]}, ones, ps0, false);
      ps1 = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{v[6], v[7]}, ones, ps1, false);
    }
    return ps0 + ps1;
  };
  // reference := max(reference, maximum of this tile); everything accumulated so far is rescaled
  auto raise_reference = [&](const f32x16& sc) {
    float mx = sc[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sc[e]);
    mx = max_across_halves(mx);
    const float m_new = fmaxf(m_run, mx * cs);
    const float a = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    mb = (m_new == -INFINITY) ? 0.f : m_new;
    l_run *= a;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o_acc[dt][e] *= a;
  };

  bf16x8 pb[2];  // the tile's probabilities, from scores_of_tile to values_of_tile
  auto scores_of_tile = [&](const int u, const bool first) {
    const char* const kb_cur = my_lds;
    // ---- S^T = K Q^T
    f32x16 sc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      const bf16x8 frag = *reinterpret_cast<const bf16x8*>(kb_cur + k_off[g >> 1] + 32 * (g & 1));
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag, qreg[g], sc, 0, 0, 0);
    }
    // causal mask: only tiles that reach past the first query's limit
    if (u * kSub + kSub - 1 > P) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = u * kSub + 16 * (e >> 3) + 8 * g2 + (e & 7);
        if (key > q_limit) sc[e] = -INFINITY;
      }
    }
    // ---- probabilities against the (stale) reference
    if (first) raise_reference(sc);
    float ps = exps(sc, pb);
    if (__any(!(ps <= kRefreshSum) || (m_run == -INFINITY && ps > 0.f))) {
      raise_reference(sc);
      ps = exps(sc, pb);
    }
    l_run += ps;
  };
  auto values_of_tile = [&]() {
    const char* const vb_cur = my_lds + kSubBytes;
    // ---- O^T += V^T P^T
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const char* vp = vb_cur + v_off[dt] + 4 * ks * kGroupBytes;
        const s16x4 lo = lds_read_tr16(reinterpret_cast<const __bf16*>(vp));
        const s16x4 hi = lds_read_tr16(reinterpret_cast<const __bf16*>(vp + kGroupBytes));
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb[ks], o_acc[dt], 0, 0, 0);
      }
  };

  // ---- the segment's tiles, one after the other; the buffers are the wave's own.  The K buffer is refilled with the
  // next tile's rows as soon as the scores are done, the V buffer as soon as the values are, so one of the two is
  // always on its way while the other is used.  Loads return in order: "all but the last eight" is exactly the older
  // of the two halves.  The waves of a workgroup read the slices of the SAME token rows, one kv-head each, and a
  // barrier per tile keeps them together: whole 2 KiB rows are fetched at about the same time (a stream of full rows
  // runs 5 % faster than the same bytes as eight independent streams of 256-byte slices).
  {
    bool first = true;
    int u = u_begin;
    Ids ids = fetch_ids(u);
    if (u < u_end) {
      issue_half(0, u, ids);
      issue_half(1, u, ids);
    }
    for (; u < u_end; ++u) {
      const bool more = u + 1 < u_end;
      const Ids ids_next = fetch_ids(u + 1);
      if (HW > 1) __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_s_waitcnt(0x0F70 | 8);  // vmcnt(8): K(u) has landed, V(u) may be on its way
      asm volatile("" ::: "memory");
      scores_of_tile(u, first);
      first = false;
      asm volatile("" ::: "memory");
      if (more) issue_half(0, u + 1, ids_next);
      if (more)
        __builtin_amdgcn_s_waitcnt(0x0F70 | 8);  // V(u) has landed, K(u+1) may be on its way
      else
        __builtin_amdgcn_s_waitcnt(0x0F70);
      asm volatile("" ::: "memory");
      values_of_tile();
      asm volatile("" ::: "memory");
      if (more) issue_half(1, u + 1, ids_next);
    }
  }

  const float l_row = sum_across_halves(l_run);
  if (whole) {
    if (q_valid)
      store_out_row(p.out + ((int64_t)(cu_s + tt) * p.n_q_heads + head) * kD, o_acc, 1.0f / l_row, g2);
  } else {
    // Two slots per range: 2 * wg for a segment that starts where the range starts (a session continued from the
    // range before), 2 * wg + 1 for one that starts inside it.  The pieces of a session are then its first one and,
    // for every further range it reaches into, that range's even slot; the wave of kv-head 0 that has the first piece
    // puts the session on the merge list.
    const int pslot = 2 * wg + (at_range_start ? 0 : 1);
    if (u_begin == 0 && kvh == 0 && lane == 0) {
      const int last_wg = (unit_end - 1) / per_wg;
      const int mi = atomicAdd(p.hdr + kHdrDecMerges, 1);  // at most one per range: the list has room for all
      if (mi < p.dec_merges_bound) p.dec_merges[mi] = MergeItem{s, 0, pslot, last_wg - wg + 1};
    }
    // The piece goes through the wave's LDS buffers into the packed layout, so that every store instruction writes
    // whole lines (the wave's own reads of the buffers are done: it has used the last tile).
    const int rows = G * N;
    const int n_floats = rows * 130;
    const int n_padded = (n_floats + 31) & ~31;
    float* const stage = reinterpret_cast<float*>(my_lds);
    if (q_valid) {
      const int r = hh * N + tt;
      float* so = stage + r * 128 + 4 * g2;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) so[32 * dt + 8 * i + j] = o_acc[dt][4 * i + j];
      if (g2 == 0) {
        stage[rows * 128 + r] = m_run;
        stage[rows * 129 + r] = l_row;
      }
    }
    if (n_floats + lane < n_padded) stage[n_floats + lane] = 0.f;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    float* part = p.dec_partials + ((int64_t)pslot * Hkv + kvh) * p.dec_slot_floats;
    for (int idx = lane; idx < n_padded; idx += 64) part[idx] = stage[idx];
    __builtin_amdgcn_wave_barrier();
  }
  }
}

// Combine the pieces of a short turn that the decode kernel cut at the boundaries of its workgroups' shares:
// out = sum_c w_c O_c / sum_c w_c l_c with w_c = 2^(m_c - max_c m_c), m_c being the piece's softmax reference in log2
// units (-inf: the piece saw no key of the row).  The first piece is in slot pslot0, piece c >= 1 in the even slot of
// the c-th workgroup after the one that wrote pslot0; pieces are added in that order.
// One workgroup per (session, kv-head); a thread per (row, d) element of the packed pieces.
template <int G>
__global__ __launch_bounds__(256) void attn_decode_merge_kernel(const MfmaParams p) {
  const int Hkv = p.n_kv_heads;
  const int mi = blockIdx.x / Hkv;
  if (mi >= min(p.hdr[kHdrDecMerges], p.dec_merges_bound)) return;
  const int kvh = blockIdx.x - mi * Hkv;
  const MergeItem m = p.dec_merges[mi];
  const int cu_s = p.cu_new_lens[m.s];
  const int N = p.cu_new_lens[m.s + 1] - cu_s;
  const int rows = G * N;
  const int first_wg = m.pslot0 >> 1;
  auto piece = [&](int c) {
    const int slot = c == 0 ? m.pslot0 : 2 * (first_wg + c);
    return p.dec_partials + ((int64_t)slot * Hkv + kvh) * p.dec_slot_floats;
  };
  for (int idx = threadIdx.x; idx < rows * 128; idx += 256) {
    const int r = idx >> 7, d = idx & 127;
    float M = -INFINITY, L = 0.f, o = 0.f;
    if (m.n_chunks <= 8) {
      // the usual case: everything is asked for at once (one trip to memory, not one for the references and another
      // for the rest), and added in piece order
      float mc[8], lc[8], oc[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float* part = piece(c < m.n_chunks ? c : 0);
        mc[c] = c < m.n_chunks ? part[rows * 128 + r] : -INFINITY;
        lc[c] = part[rows * 129 + r];
        oc[c] = part[idx];
      }
#pragma unroll
      for (int c = 0; c < 8; ++c) M = fmaxf(M, mc[c]);
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float w = (mc[c] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mc[c] - M);  // references are in log2 units
        L += w * lc[c];
        o = fmaf(w, oc[c], o);
      }
    } else {
      for (int c = 0; c < m.n_chunks; ++c) M = fmaxf(M, piece(c)[rows * 128 + r]);
      for (int c = 0; c < m.n_chunks; ++c) {
        const float* part = piece(c);
        const float mc = part[rows * 128 + r];
        const float w = (mc == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mc - M);
        L += w * part[rows * 129 + r];
        o = fmaf(w, part[idx], o);
      }
    }
    const int hh = r / N, tt = r - hh * N;
    p.out[((int64_t)(cu_s + tt) * p.n_q_heads + (kvh * G + hh)) * kD + d] = (__bf16)(o * (1.0f / L));
  }
}

// ------------------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------------------
// Tuning values with the defaults filled in (a field of symph_attn_tuning that is 0 keeps its default).
struct AttnTuning {
  int32_t slots, c_min, coarse, decode, decode_wgs;
};
static AttnTuning resolve_tuning(const symph_attn_tuning* t) {
  AttnTuning r{512, 8, 1, 1, 512};  // 512 slots: 256 compute units x 2 resident workgroups
  if (t) {
    if (t->slots > 0) r.slots = t->slots;
    if (t->c_min > 0) r.c_min = t->c_min;
    if (t->coarse != 0) r.coarse = t->coarse > 0;
    if (t->decode != 0) r.decode = t->decode > 0;
    if (t->decode_wgs > 0) r.decode_wgs = t->decode_wgs;
  }
  return r;
}

struct MfmaPlan {
  int32_t bmt, target, target_slots, c_min, coarse, units_bound, items_bound, merges_bound, pslots_bound;
  // decode kernel: whether this call runs it, its key ranges (two slots each per kv-head), room in its
  // list of sessions cut between shares
  int32_t dec_mode, dec_wgs, dec_merges_bound, dec_slot_floats;
  int64_t off_items, off_dec_s, off_dec_off, off_dec_merges, off_merge_cnt, off_partials, off_dec_partials, total_bytes;
};

static inline int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

static void lay_out(MfmaPlan& pl, int32_t n_sessions, int32_t n_kv_heads) {
  pl.items_bound = pl.units_bound + pl.pslots_bound;  // every unit once, plus one more item per chunk of a split unit
  pl.merges_bound = pl.pslots_bound / 2;              // a split unit has at least two chunks
  pl.dec_merges_bound = pl.dec_wgs;                   // at most one session starts inside a share and leaves it
  const int32_t ns = n_sessions < kSchedMaxSessions ? n_sessions : kSchedMaxSessions;  // per scheduler slice
  pl.off_items = align256(kHdrInts * 4);
  pl.off_dec_s = align256(pl.off_items + (int64_t)pl.items_bound * sizeof(WorkItem));
  pl.off_dec_off = align256(pl.off_dec_s + (int64_t)ns * 4);
  pl.off_dec_merges = align256(pl.off_dec_off + (int64_t)(ns + 1) * 4);
  pl.off_merge_cnt = align256(pl.off_dec_merges + (int64_t)pl.dec_merges_bound * sizeof(MergeItem));
  pl.off_partials = align256(pl.off_merge_cnt + (int64_t)pl.merges_bound * n_kv_heads * 4);
  pl.off_dec_partials = pl.off_partials + (int64_t)pl.pslots_bound * n_kv_heads * kPartialFloats * 4;
  pl.total_bytes = pl.off_dec_partials + (int64_t)2 * pl.dec_wgs * n_kv_heads * pl.dec_slot_floats * 4;
}

// Sizes that depend only on host-visible bounds and the tuning values, so that the workspace query and the launch
// agree.  budget_bytes > 0: the plan has to fit that many bytes; the decode kernel then gets fewer workgroups and the
// work list is cut into fewer pieces (fewer partial-result slots).  Returns false if not even the uncut list fits.
static bool make_plan(MfmaPlan& pl, int32_t n_sessions, int32_t n_q_heads, int32_t n_kv_heads,
                      int32_t total_new_tokens, int32_t max_new_len, const AttnTuning& tu, int64_t budget_bytes) {
  const int G = n_q_heads / n_kv_heads;
  pl.bmt = 128 / G;
  pl.target_slots = tu.slots < n_kv_heads ? n_kv_heads : tu.slots;  // workgroups resident at once
  pl.target = 2 * pl.target_slots;                                  // most pieces the batch is ever cut into
  pl.c_min = tu.c_min;
  pl.coarse = tu.coarse;
  pl.units_bound = total_new_tokens / pl.bmt + n_sessions;
  // A batch in which no session has more new rows than one wave holds (decode steps) takes the decode kernel: one
  // equal share of the keys per workgroup, two partial-result slots per workgroup.  Mixed batches do not: their short
  // turns are memory-bound pieces that share the CUs with the compute-bound ones inside the main kernel, which
  // measured faster than two kernels one after the other.
  pl.dec_mode = tu.decode && max_new_len >= 1 && max_new_len * G <= 32;
  // The decode kernel takes the sessions with at most max_new_len new tokens (longer ones, if the bound was understated,
  // are work items), so a piece has at most G * max_new_len rows of 130 values: slots of that size, in whole lines.
  pl.dec_slot_floats = pl.dec_mode ? ((G * max_new_len * 130 + 31) & ~31) : 0;
  // ranges of the decode kernel: one wave per (range, kv-head), as many waves as decode_wgs workgroups of four would have
  pl.dec_wgs = pl.dec_mode ? (4 * tu.decode_wgs / n_kv_heads < 1 ? 1 : 4 * tu.decode_wgs / n_kv_heads) : 0;
  // Chunks of split units: a unit is split when it has more than C tiles, C >= total tiles * kv-heads / target, so
  // there are at most target / kv-heads split units and their chunks number at most twice that.
  pl.pslots_bound = 2 * (pl.target / n_kv_heads + 1);
  lay_out(pl, n_sessions, n_kv_heads);
  if (budget_bytes <= 0 || pl.total_bytes <= budget_bytes) return true;
  // First the work list gives up its partial-result slots (in a decode step it only serves sessions longer than the
  // stated bound), then the decode kernel's ranges are halved until its pieces fit, and the work list gets back as
  // many slots as the room that is left holds.
  const int64_t slot_bytes = (int64_t)n_kv_heads * kPartialFloats * 4;
  const int32_t wanted = pl.pslots_bound;
  pl.pslots_bound = 0;
  lay_out(pl, n_sessions, n_kv_heads);
  while (pl.dec_wgs > 1 && pl.total_bytes > budget_bytes) {
    pl.dec_wgs /= 2;
    lay_out(pl, n_sessions, n_kv_heads);
  }
  const int64_t per_slot = slot_bytes + (int64_t)sizeof(WorkItem) + 4 * n_kv_heads;
  const int64_t room = budget_bytes - pl.total_bytes - 4 * 256;  // (the arrays are aligned to 256 bytes)
  if (room < 0) return false;
  const int64_t fit = room / per_slot;
  pl.pslots_bound = (int32_t)(fit < wanted ? fit : wanted) & ~1;
  const int64_t pieces = (int64_t)(pl.pslots_bound / 2) * n_kv_heads;  // (the bound above, solved for the target)
  if (pieces < pl.target) pl.target = pieces < n_kv_heads ? n_kv_heads : (int32_t)pieces;
  if (pl.target_slots > pl.target) pl.target_slots = pl.target;
  lay_out(pl, n_sessions, n_kv_heads);
  return pl.total_bytes <= budget_bytes;
}

static bool mfma_path_ok(int32_t dtype, int32_t head_dim, int32_t n_q_heads, int32_t n_kv_heads, int32_t block_size) {
  if (dtype != SYMPH_BF16 || head_dim != 128) return false;
  const int G = n_q_heads / n_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16) return false;
  return block_size >= 16 && (block_size & (block_size - 1)) == 0;
}

int64_t prefill_attn_workspace_bytes(const symph_kv_cache* c, int32_t n_sessions, int32_t n_q_heads,
                                     int32_t total_new_tokens, int32_t max_new_len, int32_t,
                                     const symph_attn_tuning* tuning) {
  if (n_q_heads % c->n_kv_heads != 0) return -1;
  if (!mfma_path_ok(c->dtype, c->head_dim, n_q_heads, c->n_kv_heads, c->block_size)) return 0;
  MfmaPlan pl;
  make_plan(pl, n_sessions, n_q_heads, c->n_kv_heads, total_new_tokens, max_new_len, resolve_tuning(tuning), 0);
  return pl.total_bytes;
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
  MfmaPlan pl;
  const AttnTuning tu = resolve_tuning(a.tuning);
  char* ws = (char*)a.workspace;
  // fit_workspace: the caller's buffer has a fixed size and the plan is made to fit it (a coarser cut of the work list)
  if (!make_plan(pl, a.n_sessions, a.n_q_heads, a.n_kv_heads, a.total_new_tokens, a.max_new_len, tu,
                 a.fit_workspace ? a.workspace_bytes : 0) ||
      !ws || a.workspace_bytes < pl.total_bytes)
    return SYMPH_EWORKSPACE;
  if (((uintptr_t)ws & 255) != 0) return SYMPH_EUNSUPPORTED;

  SchedParams sp;
  sp.cu_new_lens = a.cu_new_lens;
  sp.prefix_lens = a.prefix_lens;
  sp.n_sessions = a.n_sessions;
  sp.bmt = pl.bmt;
  sp.n_kv_heads = a.n_kv_heads;
  sp.target = pl.target;
  sp.target_slots = pl.target_slots;
  sp.coarse_ok = pl.coarse;
  sp.c_min = pl.c_min;
  sp.items_bound = pl.items_bound;
  sp.merges_bound = pl.merges_bound;
  sp.pslots_bound = pl.pslots_bound;
  sp.hdr = (int32_t*)ws;
  sp.bmt_dec = pl.dec_mode ? a.max_new_len : 0;   // (<= 32 / G in this mode)
  sp.dec_s = (int32_t*)(ws + pl.off_dec_s);
  sp.dec_off = (int32_t*)(ws + pl.off_dec_off);
  sp.items = (WorkItem*)(ws + pl.off_items);
  sp.merge_cnt = (int32_t*)(ws + pl.off_merge_cnt);
  sp.table = a.table;
  sp.table_stride = a.table_stride;
  sp.log_bs = __builtin_ctz((unsigned)a.block_size);

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
  p.merge_cnt = sp.merge_cnt;
  p.dec_s = sp.dec_s;
  p.dec_off = sp.dec_off;
  p.dec_merges = (MergeItem*)(ws + pl.off_dec_merges);
  p.dec_partials = (float*)(ws + pl.off_dec_partials);
  p.dec_slot_floats = pl.dec_slot_floats;
  p.dec_merges_bound = pl.dec_merges_bound;
  p.partials = (float*)(ws + pl.off_partials);

  const int64_t g_main = (int64_t)pl.items_bound * a.n_kv_heads;
  const int dec_hw = a.n_kv_heads % 8 == 0 ? 8 : 1;   // kv-heads (= waves) per workgroup of the decode kernel
  const int64_t g_dec = (int64_t)pl.dec_wgs * (a.n_kv_heads / dec_hw);
  const int64_t g_merge = (int64_t)pl.dec_merges_bound * a.n_kv_heads;
  if (g_main > 0x7FFFFFFFLL || g_merge > 0x7FFFFFFFLL) return SYMPH_EUNSUPPORTED;
  // The scheduler keeps one table entry per session in LDS: larger batches run as consecutive slices of sessions
  // (same stream, same workspace; the bounds of the whole batch cover every slice).
  for (int32_t s0 = 0; s0 < a.n_sessions; s0 += kSchedMaxSessions) {
    const int32_t ns = a.n_sessions - s0 < kSchedMaxSessions ? a.n_sessions - s0 : kSchedMaxSessions;
    sp.cu_new_lens = a.cu_new_lens + s0;
    sp.prefix_lens = a.prefix_lens + s0;
    sp.n_sessions = ns;
    p.cu_new_lens = sp.cu_new_lens;
    p.prefix_lens = sp.prefix_lens;
    p.table = a.table ? a.table + (int64_t)s0 * a.table_stride : nullptr;
    sp.table = p.table;
    p.n_sessions = ns;
    hipLaunchKernelGGL(attn_schedule_kernel, dim3(1), dim3(kSchedThreads), 0, stream, sp);
    // The work-item kernel runs for decode steps too.  Its list is then empty if max_new_len was a true bound; a
    // session with more new tokens than the caller stated is not a short turn for the scheduler and is computed here.
    if (a.block_size == 16)
      hipLaunchKernelGGL((attn_mfma_kernel<G, 4>), dim3((unsigned)g_main), dim3(256), 0, stream, p);
    else
      hipLaunchKernelGGL((attn_mfma_kernel<G, 0>), dim3((unsigned)g_main), dim3(256), 0, stream, p);
    if (pl.dec_mode) {
      if (dec_hw == 8) {
        if (a.block_size == 16)
          hipLaunchKernelGGL((attn_decode_kernel<G, 4, 8>), dim3((unsigned)g_dec), dim3(512), 0, stream, p);
        else
          hipLaunchKernelGGL((attn_decode_kernel<G, 0, 8>), dim3((unsigned)g_dec), dim3(512), 0, stream, p);
      } else {
        if (a.block_size == 16)
          hipLaunchKernelGGL((attn_decode_kernel<G, 4, 1>), dim3((unsigned)g_dec), dim3(64), 0, stream, p);
        else
          hipLaunchKernelGGL((attn_decode_kernel<G, 0, 1>), dim3((unsigned)g_dec), dim3(64), 0, stream, p);
      }
      hipLaunchKernelGGL((attn_decode_merge_kernel<G>), dim3((unsigned)g_merge), dim3(256), 0, stream, p);
    }
  }
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

// ------------------------------------------------------------------------------------------------------------
// matrix-core reference: nothing but MFMAs on registers, four independent accumulators per wave
// ------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void mfma_reference_kernel(int iters, float* sink) {
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(0.001f * (float)(threadIdx.x & 7));
    b[e] = (__bf16)0.5f;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) t += acc[i][3];
  if (t == -1.0f) *sink = t;  // sums of non-negative products: never taken, keeps the accumulators alive
}

int32_t launch_mfma_reference(int32_t iters, int64_t* h_flops, void* d_sink, hipStream_t stream) {
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return SYMPH_ELAUNCH;
  if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
    return SYMPH_ELAUNCH;
  const int n_wg = 2 * n_cu;
  if (h_flops) *h_flops = (int64_t)n_wg * 4 * iters * 32 * (2LL * 32 * 32 * 16);
  hipLaunchKernelGGL(mfma_reference_kernel, dim3((unsigned)n_wg), dim3(256), 0, stream, (int)iters, (float*)d_sink);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

}  // namespace symph
