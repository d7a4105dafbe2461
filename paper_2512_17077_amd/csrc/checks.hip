// Optional device-side precondition checks.  The release library documents the conditions below as the
// caller's duty (undefined behaviour if violated); a library built with -DDLLM_CHECK_PRECONDITIONS
// verifies them on the device before anything depends on them:
//   validate_offsets_kernel   cu_q, cu_kv, cu_k against the host scalars; k_b <= L_b; forced_tail <= k_b
//   validate_indices_kernel   every index of every sparse sequence inside [0, L_b) -- runs only if the
//                             offsets passed, because it walks cu_k
// Both set bits in one error word per GPU (a static device variable of this file); every other kernel of
// the library receives the word's address and returns at once when it is not zero, so a violating call
// reads and writes nothing through the bad values.  dllm_hcsa_precondition_errors() fetches and clears
// the word.  The validators read exactly the arrays the caller declared: [batch+1] offsets,
// [n_q_heads, total_k] indices, [batch] modes.
#include <mutex>

#include "common.h"
#include "precondition_rules.h"

#ifdef DLLM_CHECK_PRECONDITIONS
static __device__ uint32_t check_word_storage;
#endif

namespace dllm {

#ifdef DLLM_CHECK_PRECONDITIONS
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_mutex;
uint32_t* g_word[kMaxDevices] = {};

__global__ __launch_bounds__(256) void validate_offsets_kernel(
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ cu_k,
    const uint8_t* __restrict__ seq_mode, int32_t batch, int32_t total_q, int32_t total_kv, int32_t total_k,
    int32_t max_q, int32_t max_kv, int32_t max_k, int32_t forced_tail, uint32_t* __restrict__ word) {
  uint32_t e = 0;
  for (int b = blockIdx.x * 256 + threadIdx.x; b < batch; b += gridDim.x * 256)
    e |= dllm_rule_sequence(cu_q, cu_kv, cu_k, seq_mode, b, batch, total_q, total_kv, total_k, max_q, max_kv, max_k,
                            forced_tail);
  if (e != 0) atomicOr(word, e);
}

__global__ __launch_bounds__(256) void validate_indices_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ cu_kv, const int32_t* __restrict__ cu_k,
    const uint8_t* __restrict__ seq_mode, int32_t batch, int32_t total_k, uint32_t* __restrict__ word) {
  if (*word != 0) return;   // the offsets are not to be trusted: the lists cannot be walked
  const int h = blockIdx.y;
  uint32_t e = 0;
  for (int t = blockIdx.x * 256 + threadIdx.x; t < total_k; t += gridDim.x * 256) {
    const int b = dllm_rule_owner(cu_k, batch, t);
    e |= dllm_rule_index(idx[int64_t(h) * total_k + t], cu_kv, seq_mode, b);
  }
  if (e != 0) atomicOr(word, e);
}
}  // namespace

uint32_t* check_word() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (g_word[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(check_word_storage)) != hipSuccess) return nullptr;
    g_word[dev] = static_cast<uint32_t*>(p);
  }
  return g_word[dev];
}

hipError_t validate_inputs(const Shape& s, const int32_t* cu_q, const int32_t* cu_kv, const int32_t* cu_k,
                           const int32_t* idx, const uint8_t* seq_mode, int32_t total_k, int32_t max_k,
                           int32_t forced_tail, hipStream_t st) {
  uint32_t* word = check_word();
  if (word == nullptr) return hipErrorInvalidSymbol;
  validate_offsets_kernel<<<(s.batch + 255) / 256, 256, 0, st>>>(cu_q, cu_kv, cu_k, seq_mode, s.batch, s.total_q,
                                                                  s.total_kv, total_k, s.max_q, s.max_kv, max_k,
                                                                  forced_tail, word);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || idx == nullptr || cu_k == nullptr || total_k <= 0) return e;
  const int blocks = (total_k + 255) / 256 < 1024 ? (total_k + 255) / 256 : 1024;
  validate_indices_kernel<<<dim3(blocks, s.hq), 256, 0, st>>>(idx, cu_kv, cu_k, seq_mode, s.batch, total_k, word);
  return hipGetLastError();
}
#else
hipError_t validate_inputs(const Shape&, const int32_t*, const int32_t*, const int32_t*, const int32_t*,
                           const uint8_t*, int32_t, int32_t, int32_t, hipStream_t) {
  return hipSuccess;
}
#endif

}  // namespace dllm

extern "C" dllm_status dllm_hcsa_precondition_errors(void* hip_stream, uint32_t* errors_out) {
  if (errors_out == nullptr) return DLLM_ERR_INVALID_ARG;
  *errors_out = 0;
#ifdef DLLM_CHECK_PRECONDITIONS
  uint32_t* word = dllm::check_word();
  if (word == nullptr) return DLLM_ERR_DEVICE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint32_t host = 0;
  const uint32_t zero = 0;
  if (hipMemcpyAsync(&host, word, sizeof host, hipMemcpyDeviceToHost, st) != hipSuccess) return DLLM_ERR_DEVICE;
  if (hipMemcpyAsync(word, &zero, sizeof zero, hipMemcpyHostToDevice, st) != hipSuccess) return DLLM_ERR_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return DLLM_ERR_DEVICE;
  *errors_out = host;
  return DLLM_OK;
#else
  (void)hip_stream;
  return DLLM_ERR_UNSUPPORTED;
#endif
}
