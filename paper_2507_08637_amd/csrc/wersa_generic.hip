// Generic WERSA path: float32 arithmetic for every storage dtype, one kernel per step of
// Section 3.1 (steps 3-8), staged through caller workspace.  It covers the whole supported
// range and is the float32 product path.  Reductions are fixed-order two-pass sums.
#include "wersa_internal.h"

namespace wersa {
namespace {

#include "wersa_small_kernels.inc"

constexpr int kTileRows = 64;  // rows of one Haar tile: the largest aligned block, 2^kTileL
constexpr int kTileCols = 64;

View contiguous_view(int64_t rows, int64_t width) {
  View v;
  v.sb = rows * width;
  v.sh = 0;
  v.sn = width;
  v.H = 1;
  return v;
}

// part[slice][chunk][j] = sum over rows t of the chunk of w[slice][t] * x[slice][t][j]
template <typename T>
__global__ void colsum_partial_kernel(const T *x, View v, int n, int W, int rows_per_chunk,
                                      const float *w, float *part) {
  const int slice = blockIdx.y, chunk = blockIdx.x, chunks = gridDim.x;
  const int t0 = chunk * rows_per_chunk;
  const int t1 = min(n, t0 + rows_per_chunk);
  const T *xs = x + v.slice_base(slice);
  const int lane = threadIdx.x & 63, ph = threadIdx.x >> 6;
  __shared__ float red[4][64];
  for (int j0 = 0; j0 < W; j0 += 64) {
    const int j = j0 + lane;
    float acc = 0.f;
    if (j < W) {
      for (int t = t0 + ph; t < t1; t += 4) {
        const float xv = ld(xs + (int64_t)t * v.sn + j);
        acc += w ? w[(int64_t)slice * n + t] * xv : xv;
      }
    }
    red[ph][lane] = acc;
    __syncthreads();
    if (ph == 0 && j < W)
      part[((int64_t)slice * chunks + chunk) * W + j] =
          (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
    __syncthreads();
  }
}

// out[slice][j] = scale * sum_c part[slice][c][j]   (fixed order)
__global__ void reduce_partials_kernel(const float *part, int chunks, int64_t W, float scale,
                                       float *out) {
  const int slice = blockIdx.y;
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= W) return;
  const float *p = part + (int64_t)slice * chunks * W + j;
  float acc = 0.f;
  for (int c = 0; c < chunks; ++c) acc += p[(int64_t)c * W];
  out[(int64_t)slice * W + j] = acc * scale;
}

// In-place Haar lifting on a 64-row LDS tile, one column per lane (Appendix A equations).
// After `L` analysis levels the approximation a_L sits at rows that are multiples of 2^L and
// the level-l detail at odd multiples of 2^(l-1).
__device__ __forceinline__ void haar_analysis_tile(float (*tile)[kTileCols], int L, int c, int g) {
  const float r2 = 0.70710678118654752440f;
  for (int l = 1; l <= L; ++l) {
    const int half = 1 << (l - 1), stride = 1 << l, pairs = kTileRows >> l;
    for (int p = g; p < pairs; p += 4) {
      const int i0 = p * stride, i1 = i0 + half;
      const float a = tile[i0][c], b = tile[i1][c];
      tile[i0][c] = (a + b) * r2;
      tile[i1][c] = (a - b) * r2;
    }
    __syncthreads();
  }
}
__device__ __forceinline__ void haar_synthesis_tile(float (*tile)[kTileCols], int L, int c, int g) {
  const float r2 = 0.70710678118654752440f;
  for (int l = L; l >= 1; --l) {
    const int half = 1 << (l - 1), stride = 1 << l, pairs = kTileRows >> l;
    for (int p = g; p < pairs; p += 4) {
      const int i0 = p * stride, i1 = i0 + half;
      const float a = tile[i0][c], dt = tile[i1][c];
      tile[i0][c] = (a + dt) * r2;
      tile[i1][c] = (a - dt) * r2;
    }
    __syncthreads();
  }
}
// Band index of in-place coefficient row r: a_L at multiples of 2^L, else detail level ctz+1.
__device__ __forceinline__ int band_of_row(int r, int L) {
  const int pos = r & ((1 << L) - 1);
  return pos == 0 ? L : __builtin_ctz(pos);
}

// One level of the transform as the tile kernels see it.  Up to six analysis levels run inside a
// 64-row tile; a deeper transform (L > 6) continues on the tiles' approximation coefficients
// a_6, a signal of ceil(n / 64) rows that goes through the same kernels again (Algorithm 2's
// recursion on the approximation, 64 rows = six levels at a time).
struct HaarLevel {
  int Lt;       // analysis levels inside the tile at this stage (6 unless it is the last stage)
  int foff;     // index into F of this stage's finest detail band
  int fstride;  // L + 1: entries of F per slice
  int top;      // last stage: the tile's approximation band is a_L, gated by F[L]
};

// y = W^-1 (F (.) W x) (+ addscale * addvec[slice][j]) on 64-row x 64-column tiles.
//   approx_out != nullptr: also write the tile's a_6 to approx_out[slice][tile][j] (Lt == 6)
//   y == nullptr: stop after that (analysis only)
//   approx_in != nullptr: the tile's a_6 is replaced by approx_in[slice][tile][j] (the filtered
//   coefficient coming back from the deeper stage) before the synthesis
template <typename TIn, typename TOut>
__global__ void haar_filter_kernel(const TIn *x, View vin, TOut *y, View vout, const float *filt,
                                   const float *addvec, float addscale, int n, int d, HaarLevel lv,
                                   const float *approx_in, float *approx_out) {
  __shared__ float tile[kTileRows][kTileCols];
  __shared__ float F[kTileBands];
  const int slice = blockIdx.z, L = lv.Lt;
  const int t0 = blockIdx.x * kTileRows, j = blockIdx.y * kTileCols + (threadIdx.x & 63);
  const int c = threadIdx.x & 63, g = threadIdx.x >> 6;
  if ((int)threadIdx.x <= L)
    F[threadIdx.x] = ((int)threadIdx.x < L || lv.top) ? filt[slice * lv.fstride + lv.foff + threadIdx.x] : 1.0f;
  const TIn *xs = x + vin.slice_base(slice);
  for (int r = g; r < kTileRows; r += 4) {
    const int t = t0 + r;
    tile[r][c] = (t < n && j < d) ? ld(xs + (int64_t)t * vin.sn + j) : 0.f;
  }
  __syncthreads();
  haar_analysis_tile(tile, L, c, g);
  const int64_t aidx = ((int64_t)slice * gridDim.x + blockIdx.x) * d + j;
  if (approx_out && g == 0 && j < d) approx_out[aidx] = tile[0][c];
  if (!y) return;
  for (int r = g; r < kTileRows; r += 4) tile[r][c] *= F[band_of_row(r, L)];
  if (approx_in && g == 0 && j < d) tile[0][c] = approx_in[aidx];
  __syncthreads();
  haar_synthesis_tile(tile, L, c, g);
  TOut *ys = y + vout.slice_base(slice);
  const float add = (addvec && j < d) ? addscale * addvec[(int64_t)slice * d + j] : 0.f;
  for (int r = g; r < kTileRows; r += 4) {
    const int t = t0 + r;
    if (t < n && j < d) st(ys + (int64_t)t * vout.sn + j, tile[r][c] + add);
  }
}

// part[slice][tile][foff + band] (=, or += when accumulate) sum over the tile of
// band_i(W x) * band_i(W g) for this stage's bands; `tiles0` is the tile count of the first
// stage (the row stride of part).  The first stage of a deeper transform writes zeros into
// the bands of the later stages, which then add their sums to the rows of their own tiles.
// approx_out_x / approx_out_g: the tiles' a_6 of both operands for the next stage.
template <typename TX>
__global__ void band_dots_kernel(const TX *x, View vx, const float *gr, View vg, int n, int d,
                                 HaarLevel lv, int64_t tiles0, int accumulate, float *part,
                                 float *approx_out_x, float *approx_out_g) {
  __shared__ float tx[kTileRows][kTileCols];
  __shared__ float tg[kTileRows][kTileCols];
  __shared__ float red[4][kTileBands];
  const int slice = blockIdx.z, L = lv.Lt;
  const int t0 = blockIdx.x * kTileRows, j = blockIdx.y * kTileCols + (threadIdx.x & 63);
  const int c = threadIdx.x & 63, g = threadIdx.x >> 6;
  const TX *xs = x + vx.slice_base(slice);
  const float *gs = gr + vg.slice_base(slice);
  for (int r = g; r < kTileRows; r += 4) {
    const int t = t0 + r;
    const bool ok = (t < n && j < d);
    tx[r][c] = ok ? ld(xs + (int64_t)t * vx.sn + j) : 0.f;
    tg[r][c] = ok ? gs[(int64_t)t * vg.sn + j] : 0.f;
  }
  __syncthreads();
  haar_analysis_tile(tx, L, c, g);
  haar_analysis_tile(tg, L, c, g);
  if (approx_out_x && g == 0 && j < d) {
    const int64_t aidx = ((int64_t)slice * gridDim.x + blockIdx.x) * d + j;
    approx_out_x[aidx] = tx[0][c];
    approx_out_g[aidx] = tg[0][c];
  }
  float acc[kTileBands];
#pragma unroll
  for (int b = 0; b < kTileBands; ++b) acc[b] = 0.f;
  for (int r = g; r < kTileRows; r += 4) {
    const int band = band_of_row(r, L);
    const float pr = tx[r][c] * tg[r][c];
#pragma unroll
    for (int b = 0; b < kTileBands; ++b) acc[b] += (band == b) ? pr : 0.f;
  }
#pragma unroll
  for (int b = 0; b < kTileBands; ++b) {
    const float s = wave_sum(acc[b]);
    if (c == 0) red[g][b] = s;
  }
  __syncthreads();
  const int nb = lv.top ? L + 1 : L;   // the approximation band counts at the last stage only
  const int64_t tile_id = (int64_t)blockIdx.x * gridDim.y + blockIdx.y;
  float *row = part + ((int64_t)slice * tiles0 + tile_id) * lv.fstride;
  if (accumulate) {
    if ((int)threadIdx.x < nb)
      row[lv.foff + threadIdx.x] +=
          (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
  } else {
    for (int i = threadIdx.x; i < lv.fstride; i += blockDim.x)
      row[i] = i < nb ? (red[0][i] + red[1][i]) + (red[2][i] + red[3][i]) : 0.f;
  }
}

// Strided (B,H,n,W) tensor of dtype T  ->  contiguous float32 [slices][n][W]
template <typename T>
__global__ void gather_f32_kernel(const T *x, View v, int n, int W, int64_t total, float *y) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int j = (int)(i % W);
    const int64_t r = i / W;
    const int t = (int)(r % n);
    const int slice = (int)(r / n);
    y[i] = ld(x + v.slice_base(slice) + (int64_t)t * v.sn + j);
  }
}
// contiguous float32 [slices][n][W] (optionally divided by rowdiv[slice][t]) -> strided T
template <typename T>
__global__ void scatter_kernel(const float *x, const float *rowdiv, T *y, View v, int n, int W,
                               int64_t total) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int j = (int)(i % W);
    const int64_t r = i / W;
    const int t = (int)(r % n);
    const int slice = (int)(r / n);
    float val = x[i];
    if (rowdiv) val /= rowdiv[r];
    st(y + v.slice_base(slice) + (int64_t)t * v.sn + j, val);
  }
}

// ------------------------------------------------------------------------------------
// Batched float32 GEMM with arbitrary operand strides (covers NN / TN / NT) and split-K.
//   C[bz][s] (M x N, row-major ldc) = alpha * sum_{k in split s} A(i,k) B(k,j)  (+ ReLU first)
// ------------------------------------------------------------------------------------
struct GemmArgs {
  const float *A, *B;
  float *C;
  int M, N, K;
  int64_t sAi, sAk, sBk, sBj, ldc;
  int64_t bsA, bsB, bsC;  // batch strides
  int splits;
  int64_t splitC;         // stride between the partial results of one batch entry
  const float *alpha;     // device scalar or nullptr (= 1)
  int relu;               // apply max(.,0) before alpha
};

// 64 x 64 output tile per workgroup, 16 k per LDS stage; the four waves each own a 32 x 32 quadrant
// and accumulate it on the matrix cores in float32 (v_mfma_f32_32x32x2_f32: lane (l32, h) supplies
// A(row l32, k = h) and B(k = h, column l32) of a k-pair; accumulator register i is row
// 8 (i / 4) + 4 h + (i % 4), column l32 of the quadrant).
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs a) {
  constexpr int BM = 64, BN = 64, BK = 16;
  typedef float f32x16 __attribute__((ext_vector_type(16)));
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int bz = blockIdx.z / a.splits, sp = blockIdx.z % a.splits;
  const float *A = a.A + (int64_t)bz * a.bsA;
  const float *B = a.B + (int64_t)bz * a.bsB;
  float *C = a.C + (int64_t)bz * a.bsC + (int64_t)sp * a.splitC;
  const int i0 = blockIdx.y * BM, j0 = blockIdx.x * BN;
  int kc = (a.K + a.splits - 1) / a.splits;
  kc = (kc + BK - 1) / BK * BK;
  const int kbeg = sp * kc, kend = min(a.K, kbeg + kc);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  // Each thread moves four elements of A and four of B per stage, always the same positions of the
  // tile (lanes run along whichever index is contiguous in memory): one running pointer per element,
  // advanced by a stage, and the next stage's values are requested before the current one is used.
  const bool a_k_fast = (a.sAk == 1), b_j_fast = (a.sBj == 1);
  const float *pa[4], *pb[4];
  int ka[4], ia[4], kb[4], jb[4];
  bool oka[4], okb[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int e = tid + 256 * q;
    if (a_k_fast) { ka[q] = e & 15; ia[q] = e >> 4; } else { ia[q] = e & 63; ka[q] = e >> 6; }
    if (b_j_fast) { jb[q] = e & 63; kb[q] = e >> 6; } else { kb[q] = e & 15; jb[q] = e >> 4; }
    oka[q] = i0 + ia[q] < a.M;
    okb[q] = j0 + jb[q] < a.N;
    pa[q] = A + (int64_t)(i0 + ia[q]) * a.sAi + (int64_t)(kbeg + ka[q]) * a.sAk;
    pb[q] = B + (int64_t)(kbeg + kb[q]) * a.sBk + (int64_t)(j0 + jb[q]) * a.sBj;
  }
  float ra[4], rb[4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      ra[q] = (oka[q] && k0 + ka[q] < kend) ? *pa[q] : 0.f;
      rb[q] = (okb[q] && k0 + kb[q] < kend) ? *pb[q] : 0.f;
      pa[q] += (int64_t)BK * a.sAk;
      pb[q] += (int64_t)BK * a.sBk;
    }
  };
  if (kbeg < kend) fetch(kbeg);
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      As[ka[q]][ia[q]] = ra[q];
      Bs[kb[q]][jb[q]] = rb[q];
    }
    __syncthreads();
    if (k0 + BK < kend) fetch(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[kk + h][32 * wm + l32], Bs[kk + h][32 * wn + l32], acc, 0, 0, 0);
    __syncthreads();
  }
  const float alpha = a.alpha ? *a.alpha : 1.0f;
  const int gj = j0 + 32 * wn + l32;
  if (gj < a.N) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int gi = i0 + 32 * wm + 8 * (i >> 2) + 4 * h + (i & 3);
      if (gi >= a.M) continue;
      float val = acc[i];
      if (a.relu) val = fmaxf(val, 0.f);
      C[(int64_t)gi * a.ldc + gj] = val * alpha;
    }
  }
}

// D[slice][t] = sum_r Phi[slice][t][r] z[slice][r] + eps    (one wave per row)
__global__ void rowdot_kernel(const float *phi, const float *z, int n, int m, float eps, float *D) {
  const int slice = blockIdx.y;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= n) return;
  const float *p = phi + ((int64_t)slice * n + t) * m;
  const float *zz = z + (int64_t)slice * m;
  float acc = 0.f;
  for (int r = lane; r < m; r += 64) acc += p[r] * zz[r];
  acc = wave_sum(acc);
  if (lane == 0) D[(int64_t)slice * n + t] = acc + eps;
}

// dN = dO / D (row-wise), dD_t = -<dO_t, O_t> / D_t   (one wave per row)
template <typename T>
__global__ void prep_dn_kernel(const T *dout, const T *out, View v, const float *D, int n, int d,
                               float *dN, float *dD) {
  const int slice = blockIdx.y;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= n) return;
  const int64_t base = v.slice_base(slice) + (int64_t)t * v.sn;
  const float Dt = D[(int64_t)slice * n + t];
  float acc = 0.f;
  for (int j = lane; j < d; j += 64) {
    const float g = ld(dout + base + j);
    acc += g * ld(out + base + j);
    dN[((int64_t)slice * n + t) * d + j] = g / Dt;
  }
  acc = wave_sum(acc);
  if (lane == 0) dD[(int64_t)slice * n + t] = -acc / Dt;
}

// Output stage of Algorithm 1: O_t = (N_t - mean N_t) * rstd_t over the d columns of a row,
// rstd_t = 1 / sqrt(var N_t + eps) (biased variance), kept in D.   (one wave per row)
template <typename T>
__global__ void ln_rows_kernel(const float *N, T *out, View v, int n, int d, float eps, float *D) {
  const int slice = blockIdx.y;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= n) return;
  const float *p = N + ((int64_t)slice * n + t) * d;
  float acc = 0.f;
  for (int j = lane; j < d; j += 64) acc += p[j];
  const float mu = wave_sum(acc) / (float)d;
  acc = 0.f;
  for (int j = lane; j < d; j += 64) {
    const float e = p[j] - mu;
    acc += e * e;
  }
  const float rstd = 1.0f / sqrtf(wave_sum(acc) / (float)d + eps);
  const int64_t base = v.slice_base(slice) + (int64_t)t * v.sn;
  for (int j = lane; j < d; j += 64) st(out + base + j, (p[j] - mu) * rstd);
  if (lane == 0) D[(int64_t)slice * n + t] = rstd;
}

// Backward of that stage: dN_t = rstd_t (dO_t - mean dO_t - O_t mean(dO_t * O_t)); there is no
// normaliser, so dD = 0; sig_t = -<dO_t, O_t> rstd_t^2 carries the bandwidth gradient
// (N scales with 1 / sigma^2, and <dN_t, N_t> = <dO_t, O_t> eps rstd_t^2).
template <typename T>
__global__ void prep_ln_kernel(const T *dout, const T *out, View v, const float *D, int n, int d,
                               float *dN, float *dD, float *sig) {
  const int slice = blockIdx.y;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= n) return;
  const int64_t base = v.slice_base(slice) + (int64_t)t * v.sn;
  const float rstd = D[(int64_t)slice * n + t];
  float sg = 0.f, sgo = 0.f;
  for (int j = lane; j < d; j += 64) {
    const float g = ld(dout + base + j);
    sg += g;
    sgo += g * ld(out + base + j);
  }
  sg = wave_sum(sg);
  sgo = wave_sum(sgo);
  const float m1 = sg / (float)d, m2 = sgo / (float)d;
  for (int j = lane; j < d; j += 64)
    dN[((int64_t)slice * n + t) * d + j] = rstd * (ld(dout + base + j) - m1 - ld(out + base + j) * m2);
  if (lane == 0) {
    dD[(int64_t)slice * n + t] = 0.f;
    sig[(int64_t)slice * n + t] = -sgo * rstd * rstd;
  }
}

// R = (R + a[slice][t] * b[slice][r]) * 1[Phi > 0] * c     (a == nullptr means a = 1)
__global__ void mask_scale_kernel(float *R, const float *phi, const float *a, const float *b,
                                  const float *c_ptr, int n, int m, int64_t total) {
  const float c = *c_ptr;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int r = (int)(i % m);
    const int64_t row = i / m;  // slice * n + t
    const int slice = (int)(row / n);
    const float av = a ? a[row] : 1.0f;
    const float val = R[i] + av * b[(int64_t)slice * m + r];
    R[i] = phi[i] > 0.f ? val * c : 0.f;
  }
}

// ---------------------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------------------
int colsum_chunks(int n) {
  int c = (n + 255) / 256;
  return c < 1 ? 1 : (c > 256 ? 256 : c);
}
int gemm_splits(int n) {
  int s = n / 1024;
  return s < 1 ? 1 : (s > 64 ? 64 : s);
}
int ew_blocks(int64_t total) {
  int64_t b = (total + 255) / 256;
  return (int)(b > 65536 ? 65536 : (b < 1 ? 1 : b));
}

// Stages of the transform: stage 0 works on the n rows of the tensor, stage k + 1 on the
// ceil(n_k / 64) tile approximations of stage k; six levels per stage, the rest in the last.
constexpr int kMaxStages = 4;   // 6 + 6 + 6 + 2 levels cover kMaxL = 20
struct Stages {
  int count;
  int n[kMaxStages];
  HaarLevel lv[kMaxStages];
  int64_t off[kMaxStages];   // float offset of stage k's approximation array (k >= 1) in a deep buffer
  int64_t total;             // floats of one deep buffer
};
Stages stages_of(const wersa_desc &c) {
  Stages s{};
  const int64_t sl = (int64_t)c.B * c.H;
  int rem = c.L, rows = c.n, foff = 0, k = 0;
  int64_t off = 0;
  for (;; ++k) {
    s.n[k] = rows;
    const bool last = rem <= kTileL;
    s.lv[k] = HaarLevel{last ? rem : kTileL, foff, c.L + 1, last ? 1 : 0};
    if (last) break;
    rem -= kTileL;
    foff += kTileL;
    rows = (rows + kTileRows - 1) / kTileRows;
    s.off[k + 1] = off;
    off += sl * rows * c.d;
  }
  s.count = k + 1;
  s.total = off;
  return s;
}

struct GenericWs {
  float *scalars, *qpart, *QF, *KF, *Vf, *Of, *Phi, *R, *Spart, *zpart, *Nbuf;
  float *dN, *dD, *sig, *dS, *dz, *dDpart, *dVf, *partQ, *partK, *dF, *dlogit, *dqbar;
  float *deepA, *deepB;   // approximation arrays of the transform's stages above the first (L > 6)
  int64_t total;
};

GenericWs plan(const wersa_desc &c, int bwd, float *base) {
  GenericWs w{};
  Bump b(base);
  const int64_t sl = (int64_t)c.B * c.H, nd = sl * c.n * c.d, nm = sl * c.n * c.m;
  const int chunks = colsum_chunks(c.n), splits = gemm_splits(c.n);
  const int64_t tiles = (int64_t)((c.n + kTileRows - 1) / kTileRows) * ((c.d + kTileCols - 1) / kTileCols);
  w.scalars = b.take(64);
  w.qpart = b.take(sl * chunks * (int64_t)(c.m > c.d ? c.m : c.d));
  w.QF = b.take(nd);
  w.KF = b.take(nd);
  w.Vf = b.take(nd);
  w.Of = b.take((int64_t)2 * c.d * c.m);  // Omega in float32: the query-side matrix, then the key-side one
  w.Phi = b.take(nm);
  w.Spart = b.take(sl * splits * (int64_t)c.m * c.d);
  w.zpart = w.qpart;  // same shape family, used after qpart is consumed
  w.Nbuf = b.take(nd);
  const int64_t deep = stages_of(c).total;
  w.deepA = b.take(deep);
  if (bwd) {
    w.deepB = b.take(deep);
    w.R = b.take(nm);
    w.dN = w.Nbuf;
    w.dD = b.take(sl * c.n);
    w.sig = b.take(sl * c.n);
    w.dS = b.take(sl * (int64_t)c.m * c.d);
    w.dz = b.take(sl * c.m);
    w.dDpart = b.take(sl * chunks);
    w.dVf = b.take(nd);
    w.partQ = b.take(sl * tiles * (c.L + 1));
    w.partK = b.take(sl * tiles * (c.L + 1));
    w.dF = b.take(sl * (c.L + 1));
    w.dlogit = b.take(sl * (c.L + 1));
    w.dqbar = b.take(sl * c.d);
  }
  w.total = b.off;
  return w;
}

template <typename T>
void launch_colsum(const T *x, View v, int slices, int n, int W, const float *wt, float *part,
                   float *out, float scale, hipStream_t st) {
  const int chunks = colsum_chunks(n);
  const int rows = (n + chunks - 1) / chunks;
  WERSA_STAGE("colsum_partial_kernel", st, colsum_partial_kernel<T><<<dim3(chunks, slices), 256, 0, st>>>(x, v, n, W, rows, wt, part));
  if (out)
    WERSA_STAGE("reduce_partials_kernel", st, reduce_partials_kernel<<<dim3((W + 255) / 256, slices), 256, 0, st>>>(part, chunks, W, scale, out));
}

void launch_gemm(GemmArgs a, int batch, hipStream_t st, const char *name) {
  dim3 grid((a.N + 63) / 64, (a.M + 63) / 64, batch * a.splits);
  WERSA_STAGE(name, st, gemm_kernel<<<grid, 256, 0, st>>>(a));
}

// Omega of the query side (side 0) or the key side (side 1) in float32; the same matrix unless the
// descriptor asks for separate ones.
const float *omega_of(const wersa_desc &c, const GenericWs &w, int side) {
  return w.Of + ((c.flags & WERSA_FLAG_SEPARATE_OMEGA) && side ? (int64_t)c.d * c.m : 0);
}

// Phi = ReLU(XF Omega) * c
void launch_features(const wersa_desc &c, const float *XF, int side, const GenericWs &w, hipStream_t st) {
  GemmArgs a{};
  a.A = XF; a.B = omega_of(c, w, side); a.C = w.Phi;
  a.M = c.n; a.N = c.m; a.K = c.d;
  a.sAi = c.d; a.sAk = 1; a.sBk = c.m; a.sBj = 1; a.ldc = c.m;
  a.bsA = (int64_t)c.n * c.d; a.bsB = 0; a.bsC = (int64_t)c.n * c.m;
  a.splits = 1; a.splitC = 0; a.alpha = w.scalars; a.relu = 1;
  launch_gemm(a, c.B * c.H, st, "gemm_features");
}
// out[slice] (m x d) = Phi[slice]^T Y[slice], reduced over n by split partials
void launch_phiT_times(const wersa_desc &c, const float *Y, const GenericWs &w, float *out,
                       hipStream_t st) {
  const int splits = gemm_splits(c.n), slices = c.B * c.H;
  GemmArgs a{};
  a.A = w.Phi; a.B = Y; a.C = w.Spart;
  a.M = c.m; a.N = c.d; a.K = c.n;
  a.sAi = 1; a.sAk = c.m; a.sBk = c.d; a.sBj = 1; a.ldc = c.d;
  a.bsA = (int64_t)c.n * c.m; a.bsB = (int64_t)c.n * c.d; a.bsC = (int64_t)splits * c.m * c.d;
  a.splits = splits; a.splitC = (int64_t)c.m * c.d; a.alpha = nullptr; a.relu = 0;
  launch_gemm(a, slices, st, "gemm_phiT");
  const int64_t W = (int64_t)c.m * c.d;
  WERSA_STAGE("reduce_partials_kernel", st, reduce_partials_kernel<<<dim3((unsigned)((W + 255) / 256), slices), 256, 0, st>>>(w.Spart, splits, W, 1.0f, out));
}
// C[slice] (n x N) = A[slice] (n x K) * op(B[slice]); B given by strides
void launch_rows_gemm(const wersa_desc &c, const float *A, int K, const float *B, int64_t sBk,
                      int64_t sBj, int64_t bsB, int N, float *C, hipStream_t st) {
  GemmArgs a{};
  a.A = A; a.B = B; a.C = C;
  a.M = c.n; a.N = N; a.K = K;
  a.sAi = K; a.sAk = 1; a.sBk = sBk; a.sBj = sBj; a.ldc = N;
  a.bsA = (int64_t)c.n * K; a.bsB = bsB; a.bsC = (int64_t)c.n * N;
  a.splits = 1; a.splitC = 0; a.alpha = nullptr; a.relu = 0;
  launch_gemm(a, c.B * c.H, st, "gemm_rows");
}

dim3 tile_grid(int rows, const wersa_desc &c) {
  return dim3((rows + kTileRows - 1) / kTileRows, (c.d + kTileCols - 1) / kTileCols, c.B * c.H);
}

// y = G_F x over all stages.  `deep` holds the approximation arrays of the stages above 0
// (Stages::total floats; unused when L <= 6).
template <typename TIn, typename TOut>
void launch_filter(const wersa_desc &c, const TIn *x, View vin, TOut *y, View vout, const float *filt,
                   const float *addvec, float addscale, float *deep, hipStream_t st) {
  const Stages sg = stages_of(c);
  const int K = sg.count;
  if (K == 1) {
    WERSA_STAGE("haar_filter_kernel", st, haar_filter_kernel<TIn, TOut><<<tile_grid(c.n, c), 256, 0, st>>>(
        x, vin, y, vout, filt, addvec, addscale, c.n, c.d, sg.lv[0], nullptr, nullptr));
    return;
  }
  auto arr = [&](int k) { return deep + sg.off[k]; };
  // analysis upwards: a_6 of every tile becomes the next stage's signal
  WERSA_STAGE("haar_filter_kernel", st, haar_filter_kernel<TIn, TOut><<<tile_grid(c.n, c), 256, 0, st>>>(
      x, vin, (TOut *)nullptr, vout, filt, nullptr, 0.f, c.n, c.d, sg.lv[0], nullptr, arr(1)));
  for (int k = 1; k + 1 < K; ++k) {
    const View cvk = contiguous_view(sg.n[k], c.d);
    WERSA_STAGE("haar_filter_kernel", st, haar_filter_kernel<float, float><<<tile_grid(sg.n[k], c), 256, 0, st>>>(
        arr(k), cvk, (float *)nullptr, cvk, filt, nullptr, 0.f, sg.n[k], c.d, sg.lv[k], nullptr, arr(k + 1)));
  }
  {  // last stage: plain filter of its signal, in place
    const int k = K - 1;
    const View cvk = contiguous_view(sg.n[k], c.d);
    WERSA_STAGE("haar_filter_kernel", st, haar_filter_kernel<float, float><<<tile_grid(sg.n[k], c), 256, 0, st>>>(
        arr(k), cvk, arr(k), cvk, filt, nullptr, 0.f, sg.n[k], c.d, sg.lv[k], nullptr, nullptr));
  }
  // synthesis downwards: every tile takes its filtered a_6 from the stage above
  for (int k = K - 2; k >= 1; --k) {
    const View cvk = contiguous_view(sg.n[k], c.d);
    WERSA_STAGE("haar_filter_kernel", st, haar_filter_kernel<float, float><<<tile_grid(sg.n[k], c), 256, 0, st>>>(
        arr(k), cvk, arr(k), cvk, filt, nullptr, 0.f, sg.n[k], c.d, sg.lv[k], arr(k + 1), nullptr));
  }
  WERSA_STAGE("haar_filter_kernel", st, haar_filter_kernel<TIn, TOut><<<tile_grid(c.n, c), 256, 0, st>>>(
      x, vin, y, vout, filt, addvec, addscale, c.n, c.d, sg.lv[0], arr(1), nullptr));
}

// part[slice][tile of stage 0][band] over all stages; deep_x / deep_g hold the approximation
// arrays of the two operands.
template <typename T>
void launch_band_dots(const wersa_desc &c, const T *x, View vx, const float *g, float *part,
                      float *deep_x, float *deep_g, hipStream_t st) {
  const Stages sg = stages_of(c);
  const dim3 g0 = tile_grid(c.n, c);
  const int64_t tiles0 = (int64_t)g0.x * g0.y;
  const bool deepen = sg.count > 1;
  WERSA_STAGE("band_dots_kernel", st, band_dots_kernel<T><<<g0, 256, 0, st>>>(
      x, vx, g, contiguous_view(c.n, c.d), c.n, c.d, sg.lv[0], tiles0, 0, part,
      deepen ? deep_x + sg.off[1] : nullptr, deepen ? deep_g + sg.off[1] : nullptr));
  for (int k = 1; k < sg.count; ++k) {
    const View cvk = contiguous_view(sg.n[k], c.d);
    const bool more = k + 1 < sg.count;
    WERSA_STAGE("band_dots_kernel", st, band_dots_kernel<float><<<tile_grid(sg.n[k], c), 256, 0, st>>>(
        deep_x + sg.off[k], cvk, deep_g + sg.off[k], cvk, sg.n[k], c.d, sg.lv[k], tiles0, 1, part,
        more ? deep_x + sg.off[k + 1] : nullptr, more ? deep_g + sg.off[k + 1] : nullptr));
  }
}

template <typename T>
void launch_haar(const wersa_desc &c, const T *x, View vin, float *y, const float *filt, float *deep,
                 hipStream_t st) {
  launch_filter<T, float>(c, x, vin, y, contiguous_view(c.n, c.d), filt, nullptr, 0.f, deep, st);
}

template <typename T>
wersa_status forward_t(const wersa_desc &c, const T *q, const T *k, const T *v, const T *omega_rf,
                       const float *sigma, const float *gate_w, const float *gate_b,
                       const float *scale_w, T *out, float *saved, float *ws, hipStream_t st) {
  const GenericWs w = plan(c, 0, ws);
  const SavedLayout sv = saved_layout(c);
  const int slices = c.B * c.H;
  const View tv{c.stride_b, c.stride_h, c.stride_n, c.H};
  const int64_t nd = (int64_t)slices * c.n * c.d;
  float *S = saved + sv.S, *z = saved + sv.z, *qbar = saved + sv.qbar, *s = saved + sv.s,
        *F = saved + sv.F, *D = saved + sv.D;

  WERSA_STAGE("scalars_kernel", st, scalars_kernel<<<1, 64, 0, st>>>(sigma, c.bw_floor, c.m, w.scalars));
  // step 4: pooled query and gate
  launch_colsum<T>(q, tv, slices, c.n, c.d, nullptr, w.qpart, nullptr, 1.f, st);
  WERSA_STAGE("gate_fwd_kernel", st, gate_fwd_kernel<<<slices, 256, 0, st>>>(w.qpart, colsum_chunks(c.n), c.n, c.d, c.L, c.H, gate_w,
                                         gate_b, scale_w, qbar, s, F, nullptr, (c.flags & WERSA_FLAG_POOLED_GATE) ? 1 : 0,
                                         PooledLayout{(int64_t)c.H * colsum_chunks(c.n) * c.d, (int64_t)colsum_chunks(c.n) * c.d, c.d}));
  // steps 3, 5, 6: gated Haar filter of Q and K
  launch_haar<T>(c, q, tv, w.QF, F, w.deepA, st);
  launch_haar<T>(c, k, tv, w.KF, F, w.deepA, st);
  WERSA_STAGE("gather_f32_kernel", st, gather_f32_kernel<T><<<ew_blocks(nd), 256, 0, st>>>(v, tv, c.n, c.d, nd, w.Vf));
  {
    const int64_t om = (int64_t)c.d * c.m * ((c.flags & WERSA_FLAG_SEPARATE_OMEGA) ? 2 : 1);
    WERSA_STAGE("gather_f32_kernel", st, gather_f32_kernel<T><<<ew_blocks(om), 256, 0, st>>>(
        omega_rf, contiguous_view(c.d, c.m), c.d, c.m, om, w.Of));
  }
  // step 7 on K, then S = Phi_K^T V and z = Phi_K^T 1
  launch_features(c, w.KF, 1, w, st);
  launch_phiT_times(c, w.Vf, w, S, st);
  launch_colsum<float>(w.Phi, contiguous_view(c.n, c.m), slices, c.n, c.m, nullptr, w.zpart, z, 1.f, st);
  // step 7 on Q, then step 8
  launch_features(c, w.QF, 0, w, st);
  launch_rows_gemm(c, w.Phi, c.m, S, c.d, 1, (int64_t)c.m * c.d, c.d, w.Nbuf, st);
  if (c.flags & WERSA_FLAG_LAYERNORM) {
    WERSA_STAGE("ln_rows_kernel", st, ln_rows_kernel<T><<<dim3((c.n + 3) / 4, slices), 256, 0, st>>>(w.Nbuf, out, tv, c.n, c.d, c.eps, D));
  } else {
    WERSA_STAGE("rowdot_kernel", st, rowdot_kernel<<<dim3((c.n + 3) / 4, slices), 256, 0, st>>>(w.Phi, z, c.n, c.m, c.eps, D));
    WERSA_STAGE("scatter_kernel", st, scatter_kernel<T><<<ew_blocks(nd), 256, 0, st>>>(w.Nbuf, D, out, tv, c.n, c.d, nd));
  }
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

template <typename T>
wersa_status backward_t(const wersa_desc &c, const T *q, const T *k, const T *v, const T *omega_rf,
                        const float *sigma, const float *gate_w, const float *gate_b,
                        const float *scale_w, const T *out, const T *dout, const float *saved,
                        T *dq, T *dk, T *dv, float *dgate_w, float *dgate_b, float *dscale_w,
                        float *dsigma, float *ws, hipStream_t st) {
  (void)gate_b;
  const GenericWs w = plan(c, 1, ws);
  const SavedLayout sv = saved_layout(c);
  const int slices = c.B * c.H;
  const View tv{c.stride_b, c.stride_h, c.stride_n, c.H};
  const View cv = contiguous_view(c.n, c.d);
  const int64_t nd = (int64_t)slices * c.n * c.d, nm = (int64_t)slices * c.n * c.m;
  const float *S = saved + sv.S, *z = saved + sv.z, *qbar = saved + sv.qbar, *s = saved + sv.s,
              *F = saved + sv.F, *D = saved + sv.D;
  const int64_t md = (int64_t)c.m * c.d;

  WERSA_STAGE("scalars_kernel", st, scalars_kernel<<<1, 64, 0, st>>>(sigma, c.bw_floor, c.m, w.scalars));
  launch_haar<T>(c, q, tv, w.QF, F, w.deepA, st);
  launch_haar<T>(c, k, tv, w.KF, F, w.deepA, st);
  WERSA_STAGE("gather_f32_kernel", st, gather_f32_kernel<T><<<ew_blocks(nd), 256, 0, st>>>(v, tv, c.n, c.d, nd, w.Vf));
  {
    const int64_t om = (int64_t)c.d * c.m * ((c.flags & WERSA_FLAG_SEPARATE_OMEGA) ? 2 : 1);
    WERSA_STAGE("gather_f32_kernel", st, gather_f32_kernel<T><<<ew_blocks(om), 256, 0, st>>>(
        omega_rf, contiguous_view(c.d, c.m), c.d, c.m, om, w.Of));
  }
  const bool ln = (c.flags & WERSA_FLAG_LAYERNORM) != 0;
  // O = N / D, or O = LayerNorm(N)
  if (ln) {
    WERSA_STAGE("prep_ln_kernel", st, prep_ln_kernel<T><<<dim3((c.n + 3) / 4, slices), 256, 0, st>>>(dout, out, tv, D, c.n, c.d, w.dN, w.dD, w.sig));
  } else {
    WERSA_STAGE("prep_dn_kernel", st, prep_dn_kernel<T><<<dim3((c.n + 3) / 4, slices), 256, 0, st>>>(dout, out, tv, D, c.n, c.d, w.dN, w.dD));
  }
  {  // sum over everything of the per-row term of d sigma: dD, or sig with LayerNorm
    const int chunks = colsum_chunks(c.n), rows = (c.n + chunks - 1) / chunks;
    WERSA_STAGE("colsum_partial_kernel", st, colsum_partial_kernel<float><<<dim3(chunks, slices), 256, 0, st>>>(
        ln ? w.sig : w.dD, contiguous_view(c.n, 1), c.n, 1, rows, nullptr, w.dDpart));
  }
  // Q side: dPhi_Q = dN S^T + dD z^T ; dS = Phi_Q^T dN ; dz = Phi_Q^T dD
  launch_features(c, w.QF, 0, w, st);
  launch_rows_gemm(c, w.dN, c.d, S, 1, c.d, md, c.m, w.R, st);
  launch_phiT_times(c, w.dN, w, w.dS, st);
  launch_colsum<float>(w.Phi, contiguous_view(c.n, c.m), slices, c.n, c.m, w.dD, w.zpart, w.dz, 1.f, st);
  WERSA_STAGE("mask_scale_kernel", st, mask_scale_kernel<<<ew_blocks(nm), 256, 0, st>>>(w.R, w.Phi, w.dD, z, w.scalars, c.n, c.m, nm));
  // dQ_F = dU_Q Omega^T / sigma_eff (scale folded into R); reuse QF's buffer for the result
  launch_rows_gemm(c, w.R, c.m, omega_of(c, w, 0), 1, c.m, 0, c.d, w.QF, st);
  // K side: dPhi_K = V dS^T + 1 dz^T ; dV = Phi_K dS
  launch_features(c, w.KF, 1, w, st);
  launch_rows_gemm(c, w.Vf, c.d, w.dS, 1, c.d, md, c.m, w.R, st);
  WERSA_STAGE("mask_scale_kernel", st, mask_scale_kernel<<<ew_blocks(nm), 256, 0, st>>>(w.R, w.Phi, nullptr, w.dz, w.scalars, c.n, c.m, nm));
  launch_rows_gemm(c, w.Phi, c.m, w.dS, c.d, 1, md, c.d, w.dVf, st);
  WERSA_STAGE("scatter_kernel", st, scatter_kernel<T><<<ew_blocks(nd), 256, 0, st>>>(w.dVf, nullptr, dv, tv, c.n, c.d, nd));
  launch_rows_gemm(c, w.R, c.m, omega_of(c, w, 1), 1, c.m, 0, c.d, w.KF, st);
  // wavelet stage backward: dF from band inner products, then dX = G_F dX_F
  dim3 tgrid((c.n + kTileRows - 1) / kTileRows, (c.d + kTileCols - 1) / kTileCols, slices);
  const int64_t tiles = (int64_t)tgrid.x * tgrid.y;
  launch_band_dots<T>(c, q, tv, w.QF, w.partQ, w.deepA, w.deepB, st);
  launch_band_dots<T>(c, k, tv, w.KF, w.partK, w.deepA, w.deepB, st);
  WERSA_STAGE("gate_bwd_slice_kernel", st, gate_bwd_slice_kernel<<<slices, kGateBwdThreads, 0, st>>>(w.partQ, w.partK, tiles, c.L, c.d, c.H, s, gate_w,
                                               scale_w, w.dF, w.dlogit, w.dqbar, (c.flags & WERSA_FLAG_POOLED_GATE) ? 1 : 0));
  WERSA_STAGE("gate_bwd_params_kernel", st, gate_bwd_params_kernel<<<gate_bwd_params_blocks(c.H, c.L, c.d), 256, 0, st>>>(w.dF, w.dlogit, s, qbar, w.dDpart,
                                            slices * colsum_chunks(c.n), c.B, c.H, c.L, c.d, c.eps,
                                            w.scalars, dgate_w, dgate_b, dscale_w, dsigma));
  launch_filter<float, T>(c, w.QF, cv, dq, tv, F, w.dqbar, 1.0f / (float)c.n, w.deepA, st);
  launch_filter<float, T>(c, w.KF, cv, dk, tv, F, nullptr, 0.f, w.deepA, st);
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

}  // namespace

size_t generic_workspace_bytes(const wersa_desc &c, int for_backward) {
  return (size_t)plan(c, for_backward, nullptr).total * sizeof(float);
}

wersa_status generic_forward(const wersa_desc &c, const void *q, const void *k, const void *v,
                             const void *omega_rf, const float *sigma, const float *gate_w,
                             const float *gate_b, const float *scale_w, void *out, float *saved,
                             float *ws, hipStream_t st) {
  if (c.dtype == WERSA_F32)
    return forward_t<float>(c, (const float *)q, (const float *)k, (const float *)v,
                            (const float *)omega_rf, sigma, gate_w, gate_b, scale_w, (float *)out,
                            saved, ws, st);
  return forward_t<bf16_t>(c, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                           (const bf16_t *)omega_rf, sigma, gate_w, gate_b, scale_w, (bf16_t *)out,
                           saved, ws, st);
}

wersa_status generic_backward(const wersa_desc &c, const void *q, const void *k, const void *v,
                              const void *omega_rf, const float *sigma, const float *gate_w,
                              const float *gate_b, const float *scale_w, const void *out,
                              const void *dout, const float *saved, void *dq, void *dk, void *dv,
                              float *dgate_w, float *dgate_b, float *dscale_w, float *dsigma,
                              float *ws, hipStream_t st) {
  if (c.dtype == WERSA_F32)
    return backward_t<float>(c, (const float *)q, (const float *)k, (const float *)v,
                             (const float *)omega_rf, sigma, gate_w, gate_b, scale_w,
                             (const float *)out, (const float *)dout, saved, (float *)dq,
                             (float *)dk, (float *)dv, dgate_w, dgate_b, dscale_w, dsigma, ws, st);
  return backward_t<bf16_t>(c, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                            (const bf16_t *)omega_rf, sigma, gate_w, gate_b, scale_w,
                            (const bf16_t *)out, (const bf16_t *)dout, saved, (bf16_t *)dq,
                            (bf16_t *)dk, (bf16_t *)dv, dgate_w, dgate_b, dscale_w, dsigma, ws, st);
}

// The stage alone.  Without the approximation arrays it covers the single-stage range (L <= 6).
size_t generic_haar_filter_floats(const wersa_desc &c) { return (size_t)stages_of(c).total; }
wersa_status generic_haar_filter(const wersa_desc &c, const void *x, const float *filt, void *xf,
                                 float *deep, hipStream_t st) {
  if (c.L > kTileL && !deep) return WERSA_ERR_UNSUPPORTED;
  const View tv{c.stride_b, c.stride_h, c.stride_n, c.H};
  if (c.dtype == WERSA_F32)
    launch_filter<float, float>(c, (const float *)x, tv, (float *)xf, tv, filt, nullptr, 0.f, deep, st);
  else
    launch_filter<bf16_t, bf16_t>(c, (const bf16_t *)x, tv, (bf16_t *)xf, tv, filt, nullptr, 0.f, deep, st);
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

}  // namespace wersa
