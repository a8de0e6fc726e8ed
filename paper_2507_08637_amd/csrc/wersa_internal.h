// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/wersa.h"

namespace wersa {

constexpr int kTileL = 6;                 // Haar levels inside one 64-row tile
constexpr int kTileBands = kTileL + 1;
constexpr int kMaxL = 20;                 // deepest transform (levels above 6 run on tile approximations)
constexpr int kMaxBands = kMaxL + 1;
constexpr int kCoefStride = 24;           // block-mean coefficients per slice (levels 0 .. kMaxL, padded)
constexpr int kCoefScale = 22;            // MFMA path: slot of the slice's operand scale 2^k in its coefficient row
constexpr int kCoefCscale = 23;           // ... and of c * 2^-k, c = 1 / (sigma_eff sqrt(m))

// Strided view of a (B, H, n, d) tensor; element (b, h, t, j) at b*sb + h*sh + t*sn + j.
struct View {
  int64_t sb, sh, sn;
  int H;
  __host__ __device__ int64_t slice_base(int slice) const {
    return (int64_t)(slice / H) * sb + (int64_t)(slice % H) * sh;
  }
};

// ---- bf16 storage helpers (round to nearest even) --------------------------------------
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t x) {
  return __uint_as_float(((uint32_t)x) << 16);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float ld(const T *p);
template <> __device__ __forceinline__ float ld<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st(T *p, float v);
template <> __device__ __forceinline__ void st<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void st<bf16_t>(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// ---- saved-buffer layout (floats) -------------------------------------------------------
// MFMA path (bf16 storage, d in {64, 128}, m % 128 == 0, 16-byte aligned rows).
bool fast_supported(const wersa_desc &c);
inline bool use_fast(const wersa_desc &c) {
  return !(c.flags & WERSA_FLAG_GENERIC_PATH) && fast_supported(c);
}

struct SavedLayout {
  int64_t S, z, qbar, s, F, D, QF, KF, total;
  // MFMA path only: per-call constants and bf16 operand copies written by the forward and
  // read again by the backward (scalars, filter coefficients, Omega^T fp16, (S|z), S^T, z).
  int64_t scalars, coef, omT, Sx, ST, zb;
  // MFMA path with L > 6: sums of Q and K over 64-row tiles [S][n/64][d] and the per-tile
  // addends of the levels above 6 (same shape), kept for the backward.
  int64_t tileQ, tileK, addQ, addK;
};
inline SavedLayout saved_layout(const wersa_desc &c) {
  SavedLayout o;
  const int64_t sl = (int64_t)c.B * c.H;
  auto up = [](int64_t x) { return (x + 63) / 64 * 64; };
  int64_t off = 0;
  o.S = off;    off += up(sl * c.m * c.d);
  o.z = off;    off += up(sl * c.m);
  o.qbar = off; off += up(sl * c.d);
  o.s = off;    off += up(sl * (c.L + 1));
  o.F = off;    off += up(sl * (c.L + 1));
  o.D = off;    off += up(sl * c.n);
  o.QF = o.KF = o.scalars = o.coef = o.omT = o.Sx = o.ST = o.zb = -1;
  o.tileQ = o.tileK = o.addQ = o.addK = -1;
  if (use_fast(c)) {
    if (c.d != 64) {  // filtered Q and K in fp16, kept for the backward (head dimension 64 re-forms them from Q, K)
      o.QF = off; off += up(sl * c.n * c.d / 2);
      o.KF = off; off += up(sl * c.n * c.d / 2);
    }
    const int64_t md = (int64_t)c.m * c.d, mx = (int64_t)c.m * (c.d + 16);
    o.scalars = off; off += 64;
    o.coef = off;    off += up(sl * kCoefStride);
    o.omT = off;     off += up(md / 2 * ((c.flags & WERSA_FLAG_SEPARATE_OMEGA) ? 2 : 1));
    o.Sx = off;      off += up(sl * mx / 2);
    o.ST = off;      off += up(sl * md / 2);
    o.zb = off;      off += up(sl * c.m / 2);
    if (c.L > kTileL) {
      const int64_t tiles = sl * ((c.n + 63) / 64) * c.d;
      o.tileQ = off; off += up(tiles);
      o.tileK = off; off += up(tiles);
      o.addQ = off;  off += up(tiles);
      o.addK = off;  off += up(tiles);
    }
  }
  o.total = off;
  return o;
}

wersa_status validate_desc(const wersa_desc *desc);

// Optional event timing around kernel launches (see wersa_profile_enable in the header).
bool profiling();
void prof_begin(const char *name, hipStream_t st);
void prof_end(hipStream_t st);
// Launch `expr` (a kernel launch statement) as stage `name`.
#define WERSA_STAGE(name, st, ...)  \
  do {                               \
    ::wersa::prof_begin(name, st);   \
    __VA_ARGS__;                     \
    ::wersa::prof_end(st);           \
  } while (0)

// Generic path: float32 arithmetic for every dtype, staged through workspace. Correct for
// the whole supported range; it is the float32 product path and the fallback for bf16 shapes
// the MFMA path does not cover.
size_t generic_workspace_bytes(const wersa_desc &c, int for_backward);
wersa_status generic_forward(const wersa_desc &c, const void *q, const void *k, const void *v,
                             const void *omega_rf, const float *sigma, const float *gate_w,
                             const float *gate_b, const float *scale_w, void *out, float *saved,
                             float *ws, hipStream_t st);
wersa_status generic_backward(const wersa_desc &c, const void *q, const void *k, const void *v,
                              const void *omega_rf, const float *sigma, const float *gate_w,
                              const float *gate_b, const float *scale_w, const void *out,
                              const void *dout, const float *saved, void *dq, void *dk, void *dv,
                              float *dgate_w, float *dgate_b, float *dscale_w, float *dsigma,
                              float *ws, hipStream_t st);
size_t fast_workspace_bytes(const wersa_desc &c, int for_backward);
// Column sums of Q over 128-row blocks computed by the caller (the attention block's W^Q GEMM
// leaves them in its epilogue): sums[row block of (B*n)/128][H*d], float32.  When given to the
// MFMA path's forward, the pass over Q that pools the queries is skipped.  Needs n % 128 == 0.
struct PooledSums {
  const float *sums;    // [token rows / 128][hidden]: column sums of Q' per 128 rows
  int64_t hidden;
  const float *amax;    // [token rows / 128][hidden / kPooledMaxCols]: largest |Q'| per 128 rows and column group
};
constexpr int kPooledMaxCols = 64;
wersa_status fast_forward(const wersa_desc &c, const void *q, const void *k, const void *v,
                          const void *omega_rf, const float *sigma, const float *gate_w,
                          const float *gate_b, const float *scale_w, void *out, float *saved,
                          float *ws, hipStream_t st, const PooledSums *pooled = nullptr);
// wersa_forward after validation of the descriptor and buffers, with the optional pooled sums.
wersa_status forward_checked(const wersa_desc *desc, const void *q, const void *k, const void *v,
                             const void *omega_rf, const float *sigma, const float *gate_w,
                             const float *gate_b, const float *scale_w, void *out, void *saved,
                             void *workspace, size_t workspace_bytes, void *hip_stream,
                             const PooledSums *pooled);
wersa_status fast_backward(const wersa_desc &c, const void *q, const void *k, const void *v,
                           const void *omega_rf, const float *sigma, const float *gate_w,
                           const float *scale_w, const void *out, const void *dout,
                           const float *saved, void *dq, void *dk, void *dv, float *dgate_w,
                           float *dgate_b, float *dscale_w, float *dsigma, float *ws,
                           hipStream_t st);
// deep: approximation arrays of the stages above the first (generic_haar_filter_floats(c) floats;
// nullptr for L <= 6).
// bf16 tensors with 16-byte aligned rows, up to six levels: the stage as one streaming kernel with
// 16-byte row accesses (everything else takes generic_haar_filter)
bool fast_haar_filter_supported(const wersa_desc &c, const void *x, const void *xf);
wersa_status fast_haar_filter(const wersa_desc &c, const void *x, const float *filt, void *xf, hipStream_t st);
size_t generic_haar_filter_floats(const wersa_desc &c);
wersa_status generic_haar_filter(const wersa_desc &c, const void *x, const float *filt, void *xf,
                                 float *deep, hipStream_t st);

}  // namespace wersa
