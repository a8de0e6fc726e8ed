// C ABI entry points: argument validation and dispatch. See include/wersa.h for the contract.
#include "wersa_internal.h"

#include <mutex>

namespace wersa {

wersa_status validate_desc(const wersa_desc *c) {
  if (!c) return WERSA_ERR_INVALID_ARG;
  if (c->B < 1 || c->H < 1 || c->n < 1 || c->d < 1 || c->m < 1 || c->L < 0) return WERSA_ERR_INVALID_ARG;
  if (c->dtype != WERSA_F32 && c->dtype != WERSA_BF16) return WERSA_ERR_INVALID_ARG;
  if (!(c->eps >= 0.f) || !(c->bw_floor > 0.f)) return WERSA_ERR_INVALID_ARG;
  if (c->stride_n < c->d || c->stride_h < 0 || c->stride_b < 0) return WERSA_ERR_INVALID_ARG;
  if (c->H > 1 && c->stride_h == 0) return WERSA_ERR_INVALID_ARG;
  if (c->B > 1 && c->stride_b == 0) return WERSA_ERR_INVALID_ARG;
  if (c->L > kMaxL) return WERSA_ERR_UNSUPPORTED;
  if (c->d % 16 != 0 || c->d < 16 || c->d > 256) return WERSA_ERR_UNSUPPORTED;
  if (c->m % 16 != 0 || c->m < 16 || c->m > 4096) return WERSA_ERR_UNSUPPORTED;
  if ((int64_t)c->B * c->H > 1023) return WERSA_ERR_UNSUPPORTED;
  if ((int64_t)c->n > (int64_t)1 << 22) return WERSA_ERR_UNSUPPORTED;
  if (c->flags & ~(WERSA_FLAG_GENERIC_PATH | WERSA_FLAG_SEPARATE_OMEGA | WERSA_FLAG_POOLED_GATE |
                   WERSA_FLAG_LAYERNORM)) return WERSA_ERR_INVALID_ARG;
  return WERSA_OK;
}

static bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

// Scratch of wersa_forward_static: the forward's workspace for callers that cannot allocate.
// One copy of the array lives on every device the library's code object is loaded on, at that
// device's own address; the name below is only a host-side handle for hipGetSymbolAddress and is
// never passed to a kernel.
constexpr size_t kStaticScratchBytes = (size_t)40 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Address of the current device's copy of the scratch array (looked up once per device).
static wersa_status static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return WERSA_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return WERSA_ERR_LAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return WERSA_OK;
}

wersa_status forward_checked(const wersa_desc *desc, const void *q, const void *k, const void *v,
                                    const void *omega_rf, const float *sigma, const float *gate_w,
                                    const float *gate_b, const float *scale_w, void *out, void *saved,
                                    void *workspace, size_t workspace_bytes, void *hip_stream,
                                    const PooledSums *pooled) {
  const wersa_status vs = validate_desc(desc);
  if (vs != WERSA_OK) return vs;
  if (!q || !k || !v || !omega_rf || !sigma || !gate_w || !gate_b || !scale_w || !out || !saved)
    return WERSA_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < wersa_workspace_bytes(desc, 0) || misaligned(workspace, 256) ||
      misaligned(saved, 256))
    return WERSA_ERR_WORKSPACE;
  if (use_fast(*desc)) {
    // the MFMA path moves rows in 16-byte pieces
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(omega_rf, 16) || misaligned(out, 16))
      return WERSA_ERR_INVALID_ARG;
    return fast_forward(*desc, q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, (float *)saved,
                        (float *)workspace, (hipStream_t)hip_stream, pooled);
  }
  return generic_forward(*desc, q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, (float *)saved,
                         (float *)workspace, (hipStream_t)hip_stream);
}

}  // namespace wersa

using namespace wersa;

extern "C" {

size_t wersa_workspace_bytes(const wersa_desc *desc, int for_backward) {
  if (validate_desc(desc) != WERSA_OK) return 0;
  return use_fast(*desc) ? fast_workspace_bytes(*desc, for_backward)
                         : generic_workspace_bytes(*desc, for_backward);
}

size_t wersa_saved_bytes(const wersa_desc *desc) {
  if (validate_desc(desc) != WERSA_OK) return 0;
  return (size_t)saved_layout(*desc).total * sizeof(float);
}

int32_t wersa_selected_path(const wersa_desc *desc) {
  if (validate_desc(desc) != WERSA_OK) return -1;
  return use_fast(*desc) ? 1 : 0;
}

int64_t wersa_saved_offset(const wersa_desc *desc, int which) {
  if (validate_desc(desc) != WERSA_OK) return -1;
  const SavedLayout s = saved_layout(*desc);
  switch (which) {
    case 0: return s.S;
    case 1: return s.z;
    case 2: return s.qbar;
    case 3: return s.s;
    case 4: return s.F;
    case 5: return s.D;
    default: return -1;
  }
}

wersa_status wersa_forward(const wersa_desc *desc, const void *q, const void *k, const void *v,
                           const void *omega_rf, const float *sigma, const float *gate_w,
                           const float *gate_b, const float *scale_w, void *out, void *saved,
                           void *workspace, size_t workspace_bytes, void *hip_stream) {
  return wersa::forward_checked(desc, q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, saved, workspace,
                                workspace_bytes, hip_stream, nullptr);
}

size_t wersa_static_scratch_bytes(void) { return kStaticScratchBytes; }

wersa_status wersa_forward_static(const wersa_desc *desc, const void *q, const void *k, const void *v,
                                  const void *omega_rf, const float *sigma, const float *gate_w,
                                  const float *gate_b, const float *scale_w, void *out, void *saved,
                                  void *hip_stream) {
  const wersa_status vs = validate_desc(desc);
  if (vs != WERSA_OK) return vs;
  const size_t need = wersa_workspace_bytes(desc, 0);
  if (need == 0 || need > kStaticScratchBytes) return WERSA_ERR_WORKSPACE;   // beyond the built-in scratch
  void *ws = nullptr;
  const wersa_status ss = static_scratch(&ws);
  if (ss != WERSA_OK) return ss;
  return wersa::forward_checked(desc, q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, saved, ws,
                                kStaticScratchBytes, hip_stream, nullptr);
}

wersa_status wersa_backward(const wersa_desc *desc, const void *q, const void *k, const void *v,
                            const void *omega_rf, const float *sigma, const float *gate_w,
                            const float *gate_b, const float *scale_w, const void *out,
                            const void *dout, const void *saved, void *dq, void *dk, void *dv,
                            float *dgate_w, float *dgate_b, float *dscale_w, float *dsigma,
                            void *workspace, size_t workspace_bytes, void *hip_stream) {
  const wersa_status vs = validate_desc(desc);
  if (vs != WERSA_OK) return vs;
  if (!q || !k || !v || !omega_rf || !sigma || !gate_w || !gate_b || !scale_w || !out || !dout ||
      !saved || !dq || !dk || !dv)
    return WERSA_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < wersa_workspace_bytes(desc, 1) || misaligned(workspace, 256) ||
      misaligned(saved, 256))
    return WERSA_ERR_WORKSPACE;
  if (use_fast(*desc)) {
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(omega_rf, 16) ||
        misaligned(out, 16) || misaligned(dout, 16) || misaligned(dq, 16) || misaligned(dk, 16) || misaligned(dv, 16))
      return WERSA_ERR_INVALID_ARG;
    return fast_backward(*desc, q, k, v, omega_rf, sigma, gate_w, scale_w, out, dout,
                         (const float *)saved, dq, dk, dv, dgate_w, dgate_b, dscale_w, dsigma,
                         (float *)workspace, (hipStream_t)hip_stream);
  }
  return generic_backward(*desc, q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, dout,
                          (const float *)saved, dq, dk, dv, dgate_w, dgate_b, dscale_w, dsigma,
                          (float *)workspace, (hipStream_t)hip_stream);
}

wersa_status wersa_haar_filter(const wersa_desc *desc, const void *x, const float *filt, void *xf,
                               void *hip_stream) {
  const wersa_status vs = validate_desc(desc);
  if (vs != WERSA_OK) return vs;
  if (!x || !filt || !xf) return WERSA_ERR_INVALID_ARG;
  if (!(desc->flags & WERSA_FLAG_GENERIC_PATH) && fast_haar_filter_supported(*desc, x, xf))
    return fast_haar_filter(*desc, x, filt, xf, (hipStream_t)hip_stream);
  return generic_haar_filter(*desc, x, filt, xf, nullptr, (hipStream_t)hip_stream);
}

size_t wersa_haar_filter_workspace_bytes(const wersa_desc *desc) {
  if (validate_desc(desc) != WERSA_OK) return 0;
  return generic_haar_filter_floats(*desc) * sizeof(float);
}

wersa_status wersa_haar_filter_ws(const wersa_desc *desc, const void *x, const float *filt, void *xf,
                                  void *workspace, size_t workspace_bytes, void *hip_stream) {
  const wersa_status vs = validate_desc(desc);
  if (vs != WERSA_OK) return vs;
  if (!x || !filt || !xf) return WERSA_ERR_INVALID_ARG;
  const size_t need = generic_haar_filter_floats(*desc) * sizeof(float);
  if (need && (!workspace || workspace_bytes < need || misaligned(workspace, 256))) return WERSA_ERR_WORKSPACE;
  if (!(desc->flags & WERSA_FLAG_GENERIC_PATH) && fast_haar_filter_supported(*desc, x, xf))
    return fast_haar_filter(*desc, x, filt, xf, (hipStream_t)hip_stream);
  return generic_haar_filter(*desc, x, filt, xf, need ? (float *)workspace : nullptr, (hipStream_t)hip_stream);
}

const char *wersa_status_string(wersa_status status) {
  switch (status) {
    case WERSA_OK: return "ok";
    case WERSA_ERR_INVALID_ARG: return "invalid argument";
    case WERSA_ERR_UNSUPPORTED: return "unsupported problem shape";
    case WERSA_ERR_WORKSPACE: return "workspace or saved buffer too small or misaligned";
    case WERSA_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

int32_t wersa_version(void) { return 100; }

}  // extern "C"
