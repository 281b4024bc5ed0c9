// symph_prefix_prefill_attn_static: the attention call for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The scratch memory that symph_prefix_prefill_attn
// takes as a workspace argument is here a file-scope device array of fixed size; the kernels are the same and get its
// device address as their workspace pointer.
#include "common.h"

#include <atomic>
#include <thread>

namespace symph {

constexpr int64_t kStaticScratchBytes = 64ll << 20;
// One copy per GPU the library runs on, held until the process ends.  In host code the name is a stand-in, not a
// device address: the address is asked for once per device (below) and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];               // per device: address of that device's copy of `scratch`
static std::atomic<int> g_scratch_state[kMaxDevices];  // 0: not asked yet, 1: being asked, 2: known

// Device address of the current device's scratch array; the first call on a device does the set-up.
static int32_t static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return SYMPH_ELAUNCH;
  if (dev < 0 || dev >= kMaxDevices) return SYMPH_EUNSUPPORTED;
  for (;;) {
    int st = g_scratch_state[dev].load(std::memory_order_acquire);
    if (st == 2) {
      *out = g_scratch_ptr[dev];
      return SYMPH_OK;
    }
    if (st == 0 && g_scratch_state[dev].compare_exchange_strong(st, 1, std::memory_order_acq_rel)) {
      void* ptr = nullptr;
      const hipError_t rc = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (rc != hipSuccess || !ptr) {
        g_scratch_state[dev].store(0, std::memory_order_release);
        return SYMPH_ELAUNCH;
      }
      g_scratch_ptr[dev] = ptr;
      g_scratch_state[dev].store(2, std::memory_order_release);
      *out = ptr;
      return SYMPH_OK;
    }
    std::this_thread::yield();  // another thread is asking for this device's address
  }
}

}  // namespace symph

using namespace symph;

extern "C" {

int32_t symph_prefix_prefill_attn_static(const symph_kv_cache* cache, int32_t layer, const void* d_q,
                                         const void* d_k_new, const void* d_v_new, void* d_out,
                                         const int32_t* d_cu_new_lens, const int32_t* d_prefix_lens,
                                         const int32_t* d_block_table, int32_t table_stride, int32_t n_sessions,
                                         int32_t n_q_heads, int32_t total_new_tokens, int32_t max_new_len,
                                         int32_t max_prefix_len, float scale, void* stream) {
  void* ws = nullptr;
  const int32_t rc = static_scratch(&ws);
  if (rc != SYMPH_OK) return rc;
  // fit_workspace: the work list is cut so that its partial results fit the array; SYMPH_EWORKSPACE if the list of
  // query tiles alone does not.  Nothing is cleared here: the scheduling kernel rewrites every count, counter and the
  // page of zeros at the start of each call, and nothing else is read before it is written.
  return prefill_attn_entry(cache, layer, d_q, d_k_new, d_v_new, d_out, d_cu_new_lens, d_prefix_lens, d_block_table,
                            table_stride, n_sessions, n_q_heads, total_new_tokens, max_new_len, max_prefix_len, scale,
                            ws, kStaticScratchBytes, stream, nullptr, true);
}

}  // extern "C"
