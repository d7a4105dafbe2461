// C ABI of libdllm_hcsa: host-side argument checks, workspace plans and kernel dispatch.
// Every check happens before the first HIP call, so a rejected call launches nothing.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "common.h"

// Selection scratch of dllm_hcsa_select_static: part of the device image, so every GPU the library
// runs on holds its own copy at its own address until the process ends.  In host code the array's name
// is only a handle for hipGetSymbolAddress; the address that kernels and copies may use is looked up
// once per device, with that device current, and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[DLLM_SELECT_STATIC_BYTES];

namespace {

thread_local char g_err[320] = "";

dllm_status fail(dllm_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return st;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validates the batch descriptor and fills the kernel-side shape.
dllm_status check_batch(const dllm_batch* b, dllm::Shape* out) {
  if (b == nullptr) return fail(DLLM_ERR_INVALID_ARG, "batch descriptor is NULL");
  if (b->dtype != DLLM_F32 && b->dtype != DLLM_BF16)
    return fail(DLLM_ERR_INVALID_ARG, "dtype %d is neither DLLM_F32 nor DLLM_BF16", int(b->dtype));
  if (b->batch < 1 || b->batch > 65535) return fail(DLLM_ERR_INVALID_ARG, "batch %d outside 1..65535", b->batch);
  if (b->n_q_heads < 1 || b->n_kv_heads < 1 || b->n_q_heads > 65535)
    return fail(DLLM_ERR_INVALID_ARG, "head counts must be positive (Hq=%d, Hkv=%d)", b->n_q_heads, b->n_kv_heads);
  if (b->n_q_heads % b->n_kv_heads != 0)
    return fail(DLLM_ERR_INVALID_ARG, "n_q_heads %d is not a multiple of n_kv_heads %d", b->n_q_heads, b->n_kv_heads);
  if (b->head_dim != 64 && b->head_dim != 128)
    return fail(DLLM_ERR_INVALID_ARG, "head_dim %d is not 64 or 128", b->head_dim);
  if (!b->q || !b->k || !b->v) return fail(DLLM_ERR_INVALID_ARG, "q, k and v must be non-NULL");
  if (!b->cu_q || !b->cu_kv) return fail(DLLM_ERR_INVALID_ARG, "cu_q and cu_kv must be non-NULL");
  if (b->total_q < 0 || b->total_kv < 0 || b->max_q < 0 || b->max_kv < 0 || b->max_q > b->total_q ||
      b->max_kv > b->total_kv)
    return fail(DLLM_ERR_INVALID_ARG, "need 0 <= max_q <= total_q and 0 <= max_kv <= total_kv (got %d/%d, %d/%d)",
                b->max_q, b->total_q, b->max_kv, b->total_kv);
  const int es = b->dtype == DLLM_F32 ? 4 : 2;
  const int64_t per16 = 16 / es;
  if (b->q_stride_head < b->head_dim || b->kv_stride_head < b->head_dim || b->q_stride_tok < b->head_dim ||
      b->kv_stride_tok < b->head_dim)
    return fail(DLLM_ERR_INVALID_ARG, "strides must be at least head_dim elements");
  if (b->q_stride_tok % per16 || b->q_stride_head % per16 || b->kv_stride_tok % per16 || b->kv_stride_head % per16)
    return fail(DLLM_ERR_INVALID_ARG, "strides must be multiples of 16 bytes");
  if (!aligned16(b->q) || !aligned16(b->k) || !aligned16(b->v))
    return fail(DLLM_ERR_INVALID_ARG, "q, k and v must be 16-byte aligned");
  if (!std::isfinite(b->softmax_scale) || !(b->softmax_scale > 0.0f))
    return fail(DLLM_ERR_INVALID_ARG, "softmax_scale must be finite and positive");
  out->batch = b->batch;
  out->hq = b->n_q_heads;
  out->hkv = b->n_kv_heads;
  out->group = b->n_q_heads / b->n_kv_heads;
  out->d = b->head_dim;
  out->q_tok = b->q_stride_tok;
  out->q_head = b->q_stride_head;
  out->kv_tok = b->kv_stride_tok;
  out->kv_head = b->kv_stride_head;
  out->total_q = b->total_q;
  out->total_kv = b->total_kv;
  out->max_q = b->max_q;
  out->max_kv = b->max_kv;
  out->scale = b->softmax_scale;
  return DLLM_OK;
}

// The bf16 dense kernel addresses the rows of a 64-key tile with 32-bit byte offsets.
dllm_status check_dense_strides(const dllm_batch* b) {
  if (b->dtype == DLLM_BF16 && b->kv_stride_tok * 2 * 64 >= (int64_t(1) << 32))
    return fail(DLLM_ERR_UNSUPPORTED, "kv_stride_tok %lld is too large for the dense bf16 kernel (64 rows must span < 4 GiB)",
                static_cast<long long>(b->kv_stride_tok));
  return DLLM_OK;
}

// The bf16 gather kernel addresses the kept rows of a sequence with 32-bit byte offsets from the
// sequence's first row, computed with a 24-bit multiply.
dllm_status check_sparse_strides(const dllm_batch* b) {
  if (b->dtype != DLLM_BF16) return DLLM_OK;
  const int64_t pitch = b->kv_stride_tok * 2;
  if (pitch >= (int64_t(1) << 24) || b->max_kv > (1 << 24) || int64_t(b->max_kv) * pitch >= (int64_t(1) << 32))
    return fail(DLLM_ERR_UNSUPPORTED,
                "one sequence must have at most 2^24 K/V rows spanning < 4 GiB with a token stride < 16 MiB for the bf16 gather kernel "
                "(max_kv=%d, kv_stride_tok=%lld)", b->max_kv, static_cast<long long>(b->kv_stride_tok));
  return DLLM_OK;
}

dllm_status check_workspace(const void* ws, size_t have, size_t need) {
  if (need == 0) return DLLM_OK;
  if (ws == nullptr) return fail(DLLM_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", need);
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(DLLM_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  if (have < need) return fail(DLLM_ERR_WORKSPACE, "workspace has %zu bytes, %zu are needed", have, need);
  return DLLM_OK;
}

dllm_status device_result(hipError_t e, const char* what) {
  if (e == hipSuccess) return DLLM_OK;
  return fail(DLLM_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

constexpr int kMaxKvSelect = 32768;
constexpr int kMaxKvSelectPooled = 16384;

dllm_status check_select_scalars(const dllm_batch* b, int32_t max_k, int32_t pool_w) {
  if (max_k < 1 || max_k > b->max_kv)
    return fail(DLLM_ERR_INVALID_ARG, "max_k %d outside 1..max_kv (%d)", max_k, b->max_kv);
  if (pool_w < 1 || pool_w > 63 || pool_w % 2 == 0)
    return fail(DLLM_ERR_INVALID_ARG, "pool_w %d must be odd and within 1..63", pool_w);
  if (b->max_kv > (pool_w == 1 ? kMaxKvSelect : kMaxKvSelectPooled))
    return fail(DLLM_ERR_UNSUPPORTED, "max_kv %d exceeds the %d positions ranked per sequence (pool_w=%d)", b->max_kv,
                pool_w == 1 ? kMaxKvSelect : kMaxKvSelectPooled, pool_w);
  return DLLM_OK;
}


// Scalar and pointer checks shared by the selection entry points; fills the kernel-side shape.
dllm_status check_select_call(const dllm_batch* batch, const int32_t* cu_k, int32_t total_k, int32_t max_k,
                              int32_t pool_w, int32_t forced_tail, int32_t head_sum, const int32_t* idx_out,
                              dllm::Shape* s) {
  dllm_status st = check_batch(batch, s);
  if (st != DLLM_OK) return st;
  if ((st = check_select_scalars(batch, max_k, pool_w)) != DLLM_OK) return st;
  if (cu_k == nullptr || idx_out == nullptr) return fail(DLLM_ERR_INVALID_ARG, "cu_k and idx_out must be non-NULL");
  if (total_k < 1 || max_k > total_k)
    return fail(DLLM_ERR_INVALID_ARG, "need 1 <= max_k <= total_k (got max_k=%d, total_k=%d)", max_k, total_k);
  if (forced_tail < 0 || forced_tail > max_k)
    return fail(DLLM_ERR_INVALID_ARG, "forced_tail %d outside 0..max_k (%d)", forced_tail, max_k);
  if (head_sum != 0 && head_sum != 1) return fail(DLLM_ERR_INVALID_ARG, "head_sum must be 0 or 1 (got %d)", head_sum);
  return DLLM_OK;
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

dllm_status scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(DLLM_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(DLLM_ERR_UNSUPPORTED, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr)
      return fail(DLLM_ERR_DEVICE, "hipGetSymbolAddress(selection scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DLLM_OK;
}

}  // namespace

namespace dllm {

AttendPlan plan_attend(const Shape& s, dllm_dtype dt, int32_t max_k) {
  AttendPlan p{};
  p.chunk_rows = max_k > 0 ? max_k : 1;
  p.n_chunks = 1;
  p.max_k = max_k;
  if (dt == DLLM_BF16 && max_k > 0) {
    // Two workgroups of four waves fit a compute unit (512 slots on the chip).  With at least that many
    // (sequence, head) pairs, chunks are as long as a wave's tile list allows (2048 rows: sixteen tiles);
    // with fewer pairs, kept lists are cut finer so the chip still fills.  Chunks are multiples of the
    // 128 rows four waves take per step.
    const int64_t units = int64_t(s.batch) * s.hq;
    int64_t want = 512 / units;
    if (want < 1) want = 1;
    int64_t rows = ((max_k + want - 1) / want + 127) / 128 * 128;
    if (rows > 2048) rows = 2048;
    p.chunk_rows = int32_t(rows);
    p.n_chunks = int32_t((max_k + rows - 1) / rows);
  }
  if (p.n_chunks > 1) {
    const size_t slots = size_t(p.n_chunks) * size_t(s.total_q) * size_t(s.hq);
    p.off_po = 0;
    p.off_pm = align256(slots * s.d * sizeof(float));
    p.off_pl = p.off_pm + align256(slots * sizeof(float));
    p.bytes = p.off_pl + align256(slots * sizeof(float));
  }
  return p;
}

}  // namespace dllm

extern "C" {

const char* dllm_last_error(void) { return g_err; }

int32_t dllm_hcsa_version(void) { return 100; }

size_t dllm_hcsa_select_workspace(const dllm_batch* batch, int32_t max_k) {
  dllm::Shape s;
  if (check_batch(batch, &s) != DLLM_OK) return 0;
  (void)max_k;
  return dllm::plan_select(s).bytes;
}

dllm_status dllm_hcsa_select_ex(const dllm_batch* batch, const int32_t* cu_k, int32_t total_k, int32_t max_k,
                                int32_t pool_w, int32_t forced_tail, int32_t head_sum, int32_t* idx_out,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  dllm::Shape s;
  dllm_status st = check_select_call(batch, cu_k, total_k, max_k, pool_w, forced_tail, head_sum, idx_out, &s);
  if (st != DLLM_OK) return st;
  if ((st = check_workspace(workspace, workspace_bytes, dllm::plan_select(s).bytes)) != DLLM_OK) return st;
  g_err[0] = 0;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dllm::validate_inputs(s, batch->cu_q, batch->cu_kv, cu_k, nullptr, nullptr, total_k, max_k, forced_tail,
                                       stream);
  if (e == hipSuccess)
    e = dllm::launch_select(s, batch->dtype, batch->q, batch->k, batch->cu_q, batch->cu_kv, cu_k, total_k, max_k, pool_w,
                            forced_tail, head_sum, idx_out, workspace, stream);
  return device_result(e, "dllm_hcsa_select");
}

int32_t dllm_hcsa_set_select_form(int32_t form) { return dllm::set_select_form(form); }

int32_t dllm_hcsa_select_form_of(const dllm_batch* batch, int32_t pool_w, int32_t head_sum) {
  dllm::Shape s;
  if (check_batch(batch, &s) != DLLM_OK) return -1;
  return dllm::select_form_of(s, batch->dtype, pool_w, head_sum);
}

dllm_status dllm_hcsa_select_static(const dllm_batch* batch, const int32_t* cu_k, int32_t total_k, int32_t max_k,
                                    int32_t pool_w, int32_t forced_tail, int32_t head_sum, int32_t* idx_out,
                                    void* hip_stream) {
  dllm::Shape s;
  dllm_status st = check_select_call(batch, cu_k, total_k, max_k, pool_w, forced_tail, head_sum, idx_out, &s);
  if (st != DLLM_OK) return st;
  const size_t need = dllm::plan_select(s).bytes;
  if (need > sizeof scratch)
    return fail(DLLM_ERR_WORKSPACE,
                "this batch needs %zu bytes of selection scratch, the built-in buffer holds %zu "
                "(use dllm_hcsa_select_ex with a workspace)", need, sizeof scratch);
  void* ws = nullptr;
  if ((st = scratch_of_current_device(&ws)) != DLLM_OK) return st;
  g_err[0] = 0;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dllm::validate_inputs(s, batch->cu_q, batch->cu_kv, cu_k, nullptr, nullptr, total_k, max_k, forced_tail,
                                       stream);
  if (e == hipSuccess)
    e = dllm::launch_select(s, batch->dtype, batch->q, batch->k, batch->cu_q, batch->cu_kv, cu_k, total_k, max_k, pool_w,
                            forced_tail, head_sum, idx_out, ws, stream);
  return device_result(e, "dllm_hcsa_select_static");
}

dllm_status dllm_hcsa_select(const dllm_batch* batch, const int32_t* cu_k, int32_t total_k, int32_t max_k,
                             int32_t pool_w, int32_t* idx_out, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  return dllm_hcsa_select_ex(batch, cu_k, total_k, max_k, pool_w, 0, 0, idx_out, workspace, workspace_bytes,
                             hip_stream);
}

size_t dllm_hcsa_attend_workspace(const dllm_batch* batch, int32_t max_k) {
  dllm::Shape s;
  if (check_batch(batch, &s) != DLLM_OK || max_k < 0) return 0;
  return dllm::plan_attend(s, batch->dtype, max_k).bytes;
}

dllm_status dllm_hcsa_attend(const dllm_batch* batch, const int32_t* idx, const int32_t* cu_k, int32_t total_k,
                             int32_t max_k, const uint8_t* seq_mode, void* o, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
  dllm::Shape s;
  dllm_status st = check_batch(batch, &s);
  if (st != DLLM_OK) return st;
  if (o == nullptr) return fail(DLLM_ERR_INVALID_ARG, "o must be non-NULL");
  if (!aligned16(o)) return fail(DLLM_ERR_INVALID_ARG, "o must be 16-byte aligned");
  if (total_k < 0 || max_k < 0 || max_k > total_k || max_k > batch->max_kv)
    return fail(DLLM_ERR_INVALID_ARG, "need 0 <= max_k <= min(total_k, max_kv) (got max_k=%d, total_k=%d, max_kv=%d)",
                max_k, total_k, batch->max_kv);
  if (cu_k == nullptr && total_k > 0)
    return fail(DLLM_ERR_INVALID_ARG, "cu_k may be NULL only when total_k is 0 (got total_k=%d)", total_k);
  if (seq_mode != nullptr && (st = check_dense_strides(batch)) != DLLM_OK) return st;
  if (total_k > 0 && (st = check_sparse_strides(batch)) != DLLM_OK) return st;
  const dllm::AttendPlan plan = dllm::plan_attend(s, batch->dtype, max_k);
  if ((st = check_workspace(workspace, workspace_bytes, plan.bytes)) != DLLM_OK) return st;
  g_err[0] = 0;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dllm::validate_inputs(s, batch->cu_q, batch->cu_kv, cu_k, idx, seq_mode, total_k, max_k, 0, stream);
  // Without cu_k nothing is kept anywhere: every sequence not flagged dense gets zeros.
  if (e == hipSuccess && cu_k == nullptr)
    e = dllm::launch_zero_sparse_outputs(s, batch->dtype, batch->cu_q, seq_mode, o, stream);
  if (e != hipSuccess) return device_result(e, "dllm_hcsa_attend");
  if (batch->dtype == DLLM_F32) {
    if (cu_k != nullptr)
      e = dllm::launch_attend_f32(s, batch->q, batch->k, batch->v, batch->cu_q, batch->cu_kv, idx, cu_k, total_k,
                                  seq_mode, 0, o, stream);
    if (e == hipSuccess && seq_mode != nullptr)
      e = dllm::launch_attend_f32(s, batch->q, batch->k, batch->v, batch->cu_q, batch->cu_kv, idx, cu_k, total_k,
                                  seq_mode, 1, o, stream);
  } else {
    // dense sequences first: they are the long-running part of a mixed batch
    if (seq_mode != nullptr)
      e = dllm::launch_attend_dense_bf16(s, batch->q, batch->k, batch->v, batch->cu_q, batch->cu_kv, seq_mode, 1, o,
                                         stream);
    if (e == hipSuccess && cu_k != nullptr)
      e = dllm::launch_attend_sparse_bf16(s, plan, batch->q, batch->k, batch->v, batch->cu_q, batch->cu_kv, idx, cu_k,
                                          total_k, seq_mode, o, workspace, stream);
  }
  return device_result(e, "dllm_hcsa_attend");
}

dllm_status dllm_hcsa_pack(const dllm_batch* batch, const int32_t* idx, const int32_t* cu_k, int32_t total_k,
                           int32_t max_k, void* k_packed, void* v_packed, void* hip_stream) {
  dllm::Shape s;
  dllm_status st = check_batch(batch, &s);
  if (st != DLLM_OK) return st;
  if (idx == nullptr || cu_k == nullptr || k_packed == nullptr || v_packed == nullptr)
    return fail(DLLM_ERR_INVALID_ARG, "idx, cu_k, k_packed and v_packed must be non-NULL");
  if (!aligned16(k_packed) || !aligned16(v_packed))
    return fail(DLLM_ERR_INVALID_ARG, "k_packed and v_packed must be 16-byte aligned");
  if (total_k < 1 || max_k < 1 || max_k > total_k || max_k > batch->max_kv)
    return fail(DLLM_ERR_INVALID_ARG, "need 1 <= max_k <= min(total_k, max_kv) (got max_k=%d, total_k=%d, max_kv=%d)",
                max_k, total_k, batch->max_kv);
  g_err[0] = 0;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dllm::validate_inputs(s, batch->cu_q, batch->cu_kv, cu_k, idx, nullptr, total_k, max_k, 0, stream);
  if (e == hipSuccess)
    e = dllm::launch_pack(s, batch->dtype, batch->k, batch->v, batch->cu_kv, idx, cu_k, total_k, max_k, k_packed,
                          v_packed, stream);
  return device_result(e, "dllm_hcsa_pack");
}

size_t dllm_dense_refresh_attend_workspace(const dllm_batch* batch) {
  (void)batch;
  return 0;
}

dllm_status dllm_dense_refresh_attend(const dllm_batch* batch, void* o, void* workspace, size_t workspace_bytes,
                                      void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  dllm::Shape s;
  dllm_status st = check_batch(batch, &s);
  if (st != DLLM_OK) return st;
  if (o == nullptr) return fail(DLLM_ERR_INVALID_ARG, "o must be non-NULL");
  if (!aligned16(o)) return fail(DLLM_ERR_INVALID_ARG, "o must be 16-byte aligned");
  if ((st = check_dense_strides(batch)) != DLLM_OK) return st;
  g_err[0] = 0;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dllm::validate_inputs(s, batch->cu_q, batch->cu_kv, nullptr, nullptr, nullptr, 0, 0, 0, stream);
  if (e != hipSuccess) return device_result(e, "dllm_dense_refresh_attend");
  if (batch->dtype == DLLM_F32)
    e = dllm::launch_attend_f32(s, batch->q, batch->k, batch->v, batch->cu_q, batch->cu_kv, nullptr, nullptr, 0,
                                nullptr, 2, o, stream);
  else
    e = dllm::launch_attend_dense_bf16(s, batch->q, batch->k, batch->v, batch->cu_q, batch->cu_kv, nullptr, 2, o,
                                       stream);
  return device_result(e, "dllm_dense_refresh_attend");
}

}  // extern "C"
