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
struct MfmaParams {
  const __bf16* k_layer;
  const __bf16* v_layer;
  int64_t block_stride;
  int32_t n_blocks, block_size, n_kv_heads, n_q_heads;
  const __bf16* q;
  const __bf16* k_new;
  const __bf16* v_new;
  __bf16* out;
  const int32_t* cu_new_lens;
  const int32_t* prefix_lens;
  const int32_t* table;
  int32_t table_stride, n_sessions;
  float scale_log2e;
};

constexpr int kD = 128;         // head_dim
constexpr int kBN = 64;         // keys per tile
constexpr int kKsStride = 136;  // bf16 elements per K row in LDS (272 B: 16-byte reads of 16 rows hit 16 bank groups)
constexpr int kVtStride = 72;   // bf16 elements per V^T row in LDS (144 B)

// Row r (0..31) of the A operand of S^T = K Q^T holds key key_of_row(r) of the 32-key block, chosen so that the
// MFMA result registers 8*u .. 8*u+7 of a lane in half-wave g2 are keys 16*u + 8*g2 + 0..7.
__device__ __forceinline__ int key_of_row(int r) {
  const int j = r & 3, gg = (r >> 2) & 1, i = r >> 3;
  return 16 * (i >> 1) + 8 * gg + 4 * (i & 1) + j;
}

template <int G>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const MfmaParams p) {
  constexpr int BMT = 128 / G;  // query tokens per tile
  __shared__ __attribute__((aligned(16))) __bf16 Ks[kBN * kKsStride];
  __shared__ __attribute__((aligned(16))) __bf16 Vt[kD * kVtStride];

  const int s = blockIdx.z;
  const int kvh = blockIdx.y;
  const int cu_s = p.cu_new_lens[s];
  const int N = p.cu_new_lens[s + 1] - cu_s;
  const int t0 = blockIdx.x * BMT;
  if (t0 >= N) return;
  const int P = p.prefix_lens[s];
  const int Hkv = p.n_kv_heads;
  const int bs = p.block_size;

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
      if (q_valid) {
        qreg[st] = *reinterpret_cast<const bf16x8*>(qp + 16 * st);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qreg[st][e] = (__bf16)0.0f;
      }
    }
  }

  const int kv_len = P + min(N, t0 + BMT);  // keys any row of this tile may see
  const int n_tiles = (kv_len + kBN - 1) / kBN;
  const int total_keys = P + N;

  // staging map: thread -> 16-byte chunk c of key rows kr, kr+16, kr+32, kr+48 of the tile
  const int c = tid & 15;
  const int kr = tid >> 4;
  const int32_t* table_row = p.table + (int64_t)s * p.table_stride;

  u32x4 kreg[4], vreg[4];
  auto fetch = [&](int tile) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = tile * kBN + 16 * i + kr;
      const __bf16* kp = nullptr;
      const __bf16* vp = nullptr;
      if (key < P) {
        const int jb = key / bs;
        const int b = jb < p.table_stride ? table_row[jb] : -1;
        if (b >= 0 && b < p.n_blocks) {
          const int64_t e = (int64_t)b * p.block_stride + ((int64_t)(key - jb * bs) * Hkv + kvh) * kD + 8 * c;
          kp = p.k_layer + e;
          vp = p.v_layer + e;
        }
      } else if (key < total_keys) {
        const int64_t e = ((int64_t)(cu_s + key - P) * Hkv + kvh) * kD + 8 * c;
        kp = p.k_new + e;
        vp = p.v_new + e;
      }
      if (kp) {
        kreg[i] = *reinterpret_cast<const u32x4*>(kp);
        vreg[i] = *reinterpret_cast<const u32x4*>(vp);
      } else {
        kreg[i] = u32x4{0u, 0u, 0u, 0u};
        vreg[i] = u32x4{0u, 0u, 0u, 0u};
      }
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 16 * i + kr;
      *reinterpret_cast<u32x4*>(&Ks[row * kKsStride + 8 * c]) = kreg[i];
      const unsigned short* ve = reinterpret_cast<const unsigned short*>(&vreg[i]);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        reinterpret_cast<unsigned short*>(Vt)[(8 * c + e) * kVtStride + row] = ve[e];
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
  const int a_row = key_of_row(n);
  const int q_limit = P + tok;  // last key this query may see

  fetch(0);
  for (int tile = 0; tile < n_tiles; ++tile) {
    __syncthreads();
    stage();
    __syncthreads();
    if (tile + 1 < n_tiles) fetch(tile + 1);

    // S^T tile: 64 keys x 32 queries per wave
    f32x16 sc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sc[kb][e] = 0.f;
#pragma unroll
      for (int st = 0; st < 8; ++st) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(kb * 32 + a_row) * kKsStride + 16 * st + 8 * g2]);
        sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[st], sc[kb], 0, 0, 0);
      }
    }

    // causal mask (only tiles that reach past the first query's limit)
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

    // online softmax, one query per lane (two lanes, l and l^32, share a query and split its keys)
    float mx = sc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[kb][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * cs);
    const float mb = m_new * cs;
    float psum = 0.f;
    bf16x8 pb[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pv = __builtin_amdgcn_exp2f(fmaf(sc[kb][e], cs, -mb));
        psum += pv;
        pb[kb][e >> 3][e & 7] = (__bf16)pv;
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o_acc[dt][e] *= alpha;

    // O^T += V^T P^T
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Vt[(32 * dt + n) * kVtStride + kb * 32 + 16 * u + 8 * g2]);
          o_acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kb][u], o_acc[dt], 0, 0, 0);
        }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (q_valid) {
    const float inv = 1.0f / l_tot;
    __bf16* op = p.out + ((int64_t)(cu_s + tok) * p.n_q_heads + head) * kD;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bf16x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (__bf16)(o_acc[dt][4 * i + j] * inv);
        *reinterpret_cast<bf16x4*>(op + 32 * dt + 4 * g2 + 8 * i) = v;
      }
  }
}

// ------------------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------------------
int64_t prefill_attn_workspace_bytes(const symph_kv_cache*, int32_t, int32_t, int32_t, int32_t, int32_t) {
  return 0;
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
  MfmaParams p;
  p.k_layer = (const __bf16*)a.k_layer;
  p.v_layer = (const __bf16*)a.v_layer;
  p.block_stride = a.block_stride;
  p.n_blocks = a.n_blocks;
  p.block_size = a.block_size;
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
  constexpr int BMT = 128 / G;
  const int64_t gx = ceil_div64(a.max_new_len, BMT);
  if (gx > 0x7FFFFFFFLL || a.n_kv_heads > 65535 || a.n_sessions > 65535) return SYMPH_EUNSUPPORTED;
  hipLaunchKernelGGL((attn_mfma_kernel<G>), dim3((unsigned)gx, (unsigned)a.n_kv_heads, (unsigned)a.n_sessions),
                     dim3(256), 0, stream, p);
  return hipGetLastError() == hipSuccess ? SYMPH_OK : SYMPH_ELAUNCH;
}

int32_t launch_prefill_attn(const AttnArgs& a, hipStream_t stream) {
  const int G = a.n_q_heads / a.n_kv_heads;
  const bool aligned16 = (((uintptr_t)a.k_layer | (uintptr_t)a.v_layer | (uintptr_t)a.q | (uintptr_t)a.k_new |
                           (uintptr_t)a.v_new | (uintptr_t)a.out | (uintptr_t)(a.block_stride * 2)) & 15) == 0;
  if (a.dtype == SYMPH_BF16 && a.head_dim == 128 && aligned16) {
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
