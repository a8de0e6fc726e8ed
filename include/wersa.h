/*
 * wersa.h -- C ABI of the WERSA attention hot path for AMD MI355X (gfx950).
 *
 * WERSA (Wavelet-Enhanced Random Spectral Attention) per (batch, head) slice, with
 * Q, K, V in R^{n x d} (paper Section 3.1, steps 3-8):
 *
 *   qbar   = mean over the n rows of Q                                   (step 4, Q'_avg)
 *   F_i    = sigmoid(W_g[h] qbar + b_g[h])_i * omega_i,  i = 0..L        (step 4, F_i)
 *   X_F    = W^-1( F (.) W X )  for X in {Q, K}; W = L-level Haar DWT    (steps 3, 5, 6)
 *            band 0 = finest detail d_1 ... band L-1 = d_L, band L = approximation a_L
 *            (return order of Algorithm 2's DWT); the same F gates Q and K
 *   Phi_X  = ReLU( X_F Omega / sigma_eff ) / sqrt(m),  sigma_eff = max(sigma, bw_floor)
 *                                                    (step 7; Algorithm 1 projection lines)
 *   S      = Phi_K^T V  (m x d),   z = Phi_K^T 1  (m)                    (step 8 numerator/denominator)
 *   O      = (Phi_Q S) / (Phi_Q z + eps)                                 (step 8, attention equation)
 *
 * wersa_backward returns the gradients of a scalar loss with respect to Q, K, V, W_g, b_g,
 * omega and sigma given dO = d loss / d O (the paper states no backward; it is the derivative
 * of the forward above).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller. The library allocates
 *     nothing, frees nothing and never synchronises: work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call returns.
 *   - Tensors q, k, v, out, dout, dq, dk, dv share one layout: element (b, h, t, j) lives at
 *     b*stride_b + h*stride_h + t*stride_n + j (strides in elements, j contiguous).
 *   - omega_rf (the random matrix Omega) is d x m row-major in the tensor dtype.
 *   - Parameters and their gradients are float32: gate_w [H][L+1][d], gate_b [H][L+1],
 *     scale_w [L+1] (the per-scale weights omega), sigma [1].
 *   - Gradients are overwritten, not accumulated. dgate_w, dgate_b, dscale_w, dsigma may each
 *     be NULL to skip that output.
 *   - `saved` is written by wersa_forward and read by wersa_backward (wersa_saved_bytes).
 *     `workspace` is scratch, at least wersa_workspace_bytes; both 256-byte aligned.
 *   - All argument validation happens before anything is enqueued; on error nothing is
 *     launched. No exception or abort crosses the boundary.
 *   - No mutable global state apart from the optional profiling switch below: calls on
 *     different streams with different buffers may overlap.
 *   - Results are deterministic: reductions use fixed-order two-pass sums, no float atomics.
 */
#ifndef WERSA_H
#define WERSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  WERSA_OK = 0,
  WERSA_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive size, bad stride or enum       */
  WERSA_ERR_UNSUPPORTED = 2, /* valid problem outside the implemented range (see desc)    */
  WERSA_ERR_WORKSPACE = 3,   /* workspace_bytes too small or misaligned                    */
  WERSA_ERR_LAUNCH = 4       /* the HIP runtime refused a launch                           */
} wersa_status;

typedef enum { WERSA_F32 = 0, WERSA_BF16 = 1 } wersa_dtype;

/* desc.flags bits. By default the library picks the MFMA path (bf16 storage, fp16/bf16 matrix
 * cores, float32 accumulation) when the shape allows it: dtype bf16, d in {64, 128},
 * m % 128 == 0, strides multiples of 8 elements (any n, any L <= 20); otherwise the generic
 * float32-arithmetic path. WERSA_FLAG_GENERIC_PATH forces the generic path. */
#define WERSA_FLAG_GENERIC_PATH 1
/* Separate random matrices for the query and the key side (Algorithm 1 draws W_Q^rand and
 * W_K^rand independently; Section 3.1 step 7 uses one): omega_rf then holds two d x m row-major
 * matrices back to back, the query-side one first. */
#define WERSA_FLAG_SEPARATE_OMEGA 2
/* Gate pooled over heads (Algorithm 1: the pooled queries of all heads of a batch element are
 * concatenated and go through one linear map, giving one filter per batch element):
 * logits_i = sum_h (gate_w[h][i] . qbar_h + gate_b[h][i]), F = sigmoid(logits) * scale_w for every
 * head of that batch element. Parameter shapes are unchanged (gate_w read as the (L+1) x (H*d)
 * map in head blocks). Default (Section 3.1 step 4): each head gates itself. */
#define WERSA_FLAG_POOLED_GATE 4
/* Output stage of Algorithm 1: O = LayerNorm(phi(Q_F) (phi(K_F)^T V)) over the d columns of each
 * row (no affine parameters, biased variance, desc.eps inside the square root) in place of
 * Section 3.1's division by the normaliser. The saved per-row value is then 1 / sqrt(var + eps). */
#define WERSA_FLAG_LAYERNORM 8

/*
 * Problem descriptor (host memory, read during the call only).
 * Supported range: B, H >= 1 with B * H <= 1023 (the slices are one grid dimension of every
 * launch, shared with the split of n; larger batches are to be split over calls);
 * 1 <= n <= 2^22; 0 <= L <= 20; d % 16 == 0, 16 <= d <= 256; m % 16 == 0, 16 <= m <= 4096.
 * Anything else that is otherwise well formed returns WERSA_ERR_UNSUPPORTED.
 * MFMA path only: the filtered Q and K enter the random projection (step 7) rounded to fp16, after
 * a power-of-two scale chosen per (batch, head) slice from max|Q| and the filter of that slice
 * (ReLU is positively homogeneous, so the scale drops out exactly); inputs, bandwidth and per-scale
 * weights of any magnitude are fine as long as the filtered K of a slice stays below about 2^11
 * times the bound on its filtered Q (beyond that the fp16 operands overflow: take
 * WERSA_FLAG_GENERIC_PATH).  The block entry points take the same maxima from the epilogue of their
 * W^Q product (when n % 128 != 0 or L > 6 the core pools, and scales, by itself).
 * MFMA path only: q, k, v, omega_rf, out, dout, dq, dk, dv must be 16-byte aligned (their rows
 * are read and written in 16-byte pieces); a misaligned pointer returns WERSA_ERR_INVALID_ARG
 * before anything is enqueued (WERSA_FLAG_GENERIC_PATH takes any element-aligned pointer).
 * Any n is accepted: the Haar filter is local to aligned blocks of 2^L rows, so Algorithm 2's
 * zero padding to the next power of two and the trim after the inverse are the same as reading
 * the rows past n of the last block as zeros and not writing them (done in-kernel; the pooled
 * query averages the n real rows). L > 6 (blocks longer than one 64-row tile): six levels run
 * inside the tiles, the rest on per-tile sums.
 */
typedef struct {
  int32_t B, H, n, d, L, m;
  int32_t dtype;         /* wersa_dtype of q, k, v, omega_rf, out, dout, dq, dk, dv        */
  float eps;             /* epsilon of the normaliser (Section 3.1 step 8)                  */
  float bw_floor;        /* floor of the bandwidth (Algorithm 1: bw = max(beta, floor))     */
  int64_t stride_b, stride_h, stride_n;
  int32_t flags;         /* 0 or WERSA_FLAG_* bits                                          */
} wersa_desc;

/* Bytes of scratch needed by wersa_forward (for_backward == 0) or wersa_backward (!= 0).
 * Returns 0 if the descriptor is invalid or unsupported. */
size_t wersa_workspace_bytes(const wersa_desc *desc, int for_backward);

/* Bytes of the buffer that carries S, z, qbar, the gate activations, F and the normaliser D
 * from forward to backward. Returns 0 if the descriptor is invalid or unsupported. */
size_t wersa_saved_bytes(const wersa_desc *desc);

/* Forward pass (Section 3.1 steps 3-8). Writes out (B,H,n,d) and saved. */
wersa_status wersa_forward(const wersa_desc *desc, const void *q, const void *k, const void *v,
                           const void *omega_rf, const float *sigma, const float *gate_w,
                           const float *gate_b, const float *scale_w, void *out, void *saved,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * wersa_forward for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same computation with the workspace
 * taken from a scratch array built into the library (device memory, wersa_static_scratch_bytes()
 * = 40 MiB per GPU, held from the first use until the process ends).  The caller still passes
 * inputs, `out` and `saved`; the call allocates nothing and never synchronises.  A problem whose
 * wersa_workspace_bytes(desc, 0) exceeds the scratch returns WERSA_ERR_WORKSPACE before anything is
 * enqueued (the MFMA-path forward needs 17-35 MiB at the benchmark shapes, so those fit; deeper
 * transforms than six levels at long n and large generic-path problems do not).  Every call on a
 * GPU shares that GPU's array, whose contents are scratch (nothing in it needs to start at zero):
 * calls that overlap in time on one GPU, on any streams, race; calls on different GPUs do not.
 * The device that is current at the call must be the one that holds the tensors.
 */
size_t wersa_static_scratch_bytes(void);
wersa_status wersa_forward_static(const wersa_desc *desc, const void *q, const void *k, const void *v,
                                  const void *omega_rf, const float *sigma, const float *gate_w,
                                  const float *gate_b, const float *scale_w, void *out, void *saved,
                                  void *hip_stream);

/* Backward pass: derivative of wersa_forward. `out` and `saved` are those of the matching
 * forward call on the same inputs. */
wersa_status wersa_backward(const wersa_desc *desc, const void *q, const void *k, const void *v,
                            const void *omega_rf, const float *sigma, const float *gate_w,
                            const float *gate_b, const float *scale_w, const void *out,
                            const void *dout, const void *saved, void *dq, void *dk, void *dv,
                            float *dgate_w, float *dgate_b, float *dscale_w, float *dsigma,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Stage entry point: the gated Haar filter alone, X_F = W^-1(F (.) W X) (Section 3.1 steps
 * 3, 5, 6; Appendix A equations) for one tensor x laid out like q, with per-slice filter
 * coefficients filt [B*H][L+1] (float32, device). Output xf has the same layout and dtype.
 * It takes no workspace and covers L <= 6; a deeper transform returns WERSA_ERR_UNSUPPORTED here
 * (wersa_haar_filter_ws takes it).
 */
wersa_status wersa_haar_filter(const wersa_desc *desc, const void *x, const float *filt,
                               void *xf, void *hip_stream);

/*
 * The same stage for every L the library takes (Appendix A: L = O(log n)). Levels above 6 run
 * on the approximation coefficients of the 64-row tiles, which live in `workspace` (device
 * memory owned by the caller, 256-byte aligned, at least wersa_haar_filter_workspace_bytes(desc)
 * bytes; 0 bytes and a NULL pointer are fine for L <= 6). Contents of the workspace are scratch.
 * Errors as for wersa_forward; a workspace that is too small or misaligned returns
 * WERSA_ERR_WORKSPACE before anything is enqueued.
 */
size_t wersa_haar_filter_workspace_bytes(const wersa_desc *desc);
wersa_status wersa_haar_filter_ws(const wersa_desc *desc, const void *x, const float *filt,
                                  void *xf, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/*
 * Attention block around the core (Section 3.1 steps 1-2: Q' = X W^Q, K' = X W^K, V' = X W^V,
 * split into H heads of width d; Algorithm 1's last line: merged heads times W_out):
 *   Y = merge_heads( WERSA( split(X W^Q), split(X W^K), split(X W^V) ) ) W^out
 * x, y, dy, dx are dense (B, n, hidden) with hidden = H*d in bf16; head h owns columns
 * [h*d, (h+1)*d) and is addressed by stride (nothing is transposed); the four weights are
 * hidden x hidden row-major [in][out] in bf16; their gradients are float32 [in][out],
 * overwritten. The stride fields of desc are ignored. Supported: dtype bf16, hidden % 256 == 0,
 * (B*n) % 256 == 0, and the core's own limits; otherwise WERSA_ERR_UNSUPPORTED.
 * `saved` (wersa_block_saved_bytes) carries Q', K', V', the merged head outputs A and the
 * core's saved buffer from forward to backward; `workspace` (wersa_block_workspace_bytes) is
 * scratch. The other conventions are those of wersa_forward / wersa_backward; the core
 * parameter gradients may be NULL, the weight gradients may not.
 */
size_t wersa_block_workspace_bytes(const wersa_desc *desc, int for_backward);
size_t wersa_block_saved_bytes(const wersa_desc *desc);

wersa_status wersa_block_forward(const wersa_desc *desc, const void *x, const void *wq,
                                 const void *wk, const void *wv, const void *wo,
                                 const void *omega_rf, const float *sigma, const float *gate_w,
                                 const float *gate_b, const float *scale_w, void *y, void *saved,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

wersa_status wersa_block_backward(const wersa_desc *desc, const void *x, const void *wq,
                                  const void *wk, const void *wv, const void *wo,
                                  const void *omega_rf, const float *sigma, const float *gate_w,
                                  const float *gate_b, const float *scale_w, const void *dy,
                                  const void *saved, void *dx, float *dwq, float *dwk, float *dwv,
                                  float *dwo, float *dgate_w, float *dgate_b, float *dscale_w,
                                  float *dsigma, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/* Byte offsets of the pieces inside the block's `saved`, for tests and tools: which = 0 Q',
 * 1 K', 2 V', 3 A (each bf16 (B, n, hidden)), 4 the core's saved buffer. -1 on a bad argument. */
int64_t wersa_block_saved_offset(const wersa_desc *desc, int which);

/* Byte offsets inside the backward `workspace` of the intermediate gradients left there by
 * wersa_block_backward, for tests and tools: which = 0 dA, 1 dQ', 2 dK', 3 dV' (each bf16
 * (B, n, hidden)). -1 on a bad argument. */
int64_t wersa_block_workspace_offset(const wersa_desc *desc, int which);

/* 1 if this descriptor runs on the MFMA path, 0 if on the generic path, -1 if rejected. */
int32_t wersa_selected_path(const wersa_desc *desc);

/* Offsets (in floats) of the pieces inside `saved`, for tests and tools:
 * which = 0 S [B*H][m][d], 1 z [B*H][m], 2 qbar [B*H][d], 3 gate sigmoid s [B*H][L+1],
 * 4 F [B*H][L+1], 5 D [B*H][n]. Returns -1 on a bad argument. */
int64_t wersa_saved_offset(const wersa_desc *desc, int which);

/*
 * Optional per-kernel timing for benchmarks and tools (off by default; the only mutable
 * library state, not thread-safe). While enabled, each kernel launch is bracketed by a HIP
 * event pair on the caller's stream. wersa_profile_collect waits for the recorded events,
 * sums the elapsed time per kernel name, clears the recording and returns the number of
 * distinct names; wersa_profile_get copies entry `index` (0 on success, 1 on bad argument).
 * wersa_profile_only restricts the bracketing to launches of one kernel name (NULL or "" =
 * every launch), so that timing one kernel does not put event records between all the others.
 */
void wersa_profile_enable(int on);
void wersa_profile_only(const char *name);
void wersa_profile_reset(void);
int32_t wersa_profile_collect(void);
int32_t wersa_profile_get(int32_t index, char *name, int32_t name_len, double *total_ms,
                          int32_t *launches);

/*
 * Reference microbenchmarks for benchmarks and tools: what this device sustains, measured in the
 * calling process, next to the nominal peaks.  Both enqueue on hip_stream, WAIT for the result and
 * return it (-1.0 on a bad argument or a failed launch).
 * wersa_peak_copy: a plain streaming copy of `bytes` (multiple of 16; dst, src device pointers,
 * 16-byte aligned, not overlapping) repeated `reps` times; returns GB/s, read plus written.
 * wersa_peak_mfma: `reps` launches of a loop of independent v_mfma_f32_32x32x16_bf16 on every
 * compute unit, operands in registers; returns TFLOP/s.  `sink` is one float of device memory
 * (never written in practice).
 */
double wersa_peak_copy(void *dst, const void *src, size_t bytes, int32_t reps, void *hip_stream);
double wersa_peak_mfma(float *sink, int32_t reps, void *hip_stream);

const char *wersa_status_string(wersa_status status);

/* Library version, major*10000 + minor*100 + patch. */
int32_t wersa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WERSA_H */
