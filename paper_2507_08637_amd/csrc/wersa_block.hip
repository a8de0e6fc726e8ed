// Attention block around the WERSA core (Section 3.1 steps 1-2: Q' = X W^Q, K' = X W^K,
// V' = X W^V, split into heads; Algorithm 1's closing line: merged heads times W_out) and its
// backward.  The projections are plain dense contractions over hidden = H*d: one bf16 MFMA
// GEMM kernel (float32 accumulation) in two operand forms,
//   NT  C[M][N] = sum_s A_s[M][K] B_s[N][K]^T   (both operands contiguous along K; up to three
//       (A, B) pairs summed, which gives dX = dQ' W^Q^T + dK' W^K^T + dV' W^V^T in one pass)
//   TN  C[M][N] = A[K][M]^T B[K][N]            (both operands contiguous across K: the weight
//       gradients X^T dQ' ...; split over K into float32 partials, reduced in fixed order)
// Heads are never transposed: the core reads and writes (B, n, H*d) through its strides.
#include "wersa_internal.h"

namespace wersa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 256, BN = 256, BK = 64;   // workgroup tile
constexpr int LS = BK + 8;                   // NT form: LDS tiles [row][k], row stride (elements)
constexpr int LT = BM + 32;                  // TN form: LDS tiles [k][row]; 576-byte rows put four
                                             // consecutive k rows into different bank quarters
constexpr int kMaxSrc = 3;
constexpr int kMaxSplit = 32;

// MFMA operand (row or column l32 = lane % 32, k = 8 h + q) out of a tile stored [k][row] in LDS,
// through the transposing LDS read of gfx950 (ds_read_b64_tr_b16): within each group of 16
// lanes, lane i passes the address of four consecutive 16-bit values, taken as row i / 4,
// columns 4 (i % 4) .. + 3 of a 4 x 16 block, and receives column i of that block.  (Lane
// mapping checked on the GPU with an index-valued LDS array.)  `tile` points at (k row 0, first
// row of the 32-row operand tile); krow is this lane's first k.
__device__ __forceinline__ bf16x8 lds_operand_tr(const bf16_t *tile, int krow, int lane) {
  const int i16 = lane & 15, grp = (lane >> 4) & 1;
  const bf16_t *p0 = tile + (krow + (i16 >> 2)) * LT + 16 * grp + 4 * (i16 & 3);
  typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p0);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0 + 4 * LT));
  s16x8 r;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    r[q] = lo[q];
    r[4 + q] = hi[q];
  }
  return __builtin_bit_cast(bf16x8, r);
}

struct GemmSrc {
  const bf16_t *a[kMaxSrc];
  const bf16_t *b[kMaxSrc];
  int count;
};

__device__ __forceinline__ bf16_t to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

// TRANS = false: NT form, A [M][K] (lda), B [N][K] (ldb).  TRANS = true: TN form, A [K][M] (lda),
// B [K][N] (ldb).  OUT_F32: float32 output at C + split * M * ldc (split = this workgroup's K
// range), else bf16 output.  M % 256 == 0, N % 256 == 0, every K range a multiple of 64.
// NW waves: 4 (2 x 2 waves of 128 x 128) or 8 (2 x 4 waves of 128 x 64, two waves per SIMD).
// Logical tile ids are dealt to the eight XCDs in contiguous runs (workgroup w runs on XCD
// w % 8), n fastest within a run, so that the workgroups sharing an A panel share an L2.
template <bool TRANS, bool OUT_F32, int NW>
// colsum (bf16 output form, may be nullptr): float32 [M / 128][N], the column sums of each wave's
// 128 output rows from the float32 accumulators; the block uses them as the pooled-query partial
// sums of Q' = X W^Q (Section 3.1 step 4) instead of a separate pass over Q'.
// colmax (with colsum): float32 [M / 128][N / 64], the largest |accumulator| of each wave's 128 rows x
// 64 columns; the core derives the fp16 operand scale of a (batch, head) slice from them.
__global__ __launch_bounds__(64 * NW, 1) void gemm_bf16_kernel(GemmSrc src, int lda, int ldb, void *Cout,
                                                              int ldc, int M, int N, int K, int k_chunk,
                                                              int splits, float *colsum, float *colmax) {
  constexpr int NT = 64 * NW;
  constexpr int WN = NW / 2;            // waves along n
  constexpr int TN = 8 / WN;            // 32-column tiles per wave: 4 or 2
  constexpr int PPT = 2048 / NT;        // 16-byte pieces per thread and operand per k-step
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *At = reinterpret_cast<bf16_t *>(smem_raw);          // [2][BM][LS]
  bf16_t *Bt = At + 2 * BM * LS;                              // [2][BN][LS]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int tiles_n = N / BN, tiles = (M / BM) * tiles_n, total = tiles * splits;
  const int per = (total + 7) / 8;
  const int lt = (blockIdx.x % 8) * per + blockIdx.x / 8;
  if (lt >= total) return;
  const int split = lt / tiles, tile = lt % tiles;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const int k_begin = split * k_chunk, k_end = min(K, k_begin + k_chunk);
  const int steps_per_src = (k_end - k_begin) / BK, steps = steps_per_src * src.count;
  const int wm = (wave / WN) * 128, wn = (wave % WN) * (32 * TN);

  f32x16 acc[4][TN];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u16x8 ra[PPT], rb[PPT];
  auto fetch = [&](int s) {
    const int which = s / steps_per_src, k0 = k_begin + (s % steps_per_src) * BK;
    const bf16_t *A = src.a[which], *B = src.b[which];
    if (!TRANS) {   // 256 rows x 8 pieces of 16 bytes along K, row-major
#pragma unroll
      for (int i = 0; i < PPT; ++i) {
        const int e = tid + NT * i, r = e >> 3, cc = e & 7;
        ra[i] = *reinterpret_cast<const u16x8 *>(A + (int64_t)(m0 + r) * lda + k0 + cc * 8);
        rb[i] = *reinterpret_cast<const u16x8 *>(B + (int64_t)(n0 + r) * ldb + k0 + cc * 8);
      }
    } else {        // 64 k rows x 32 pieces of 16 bytes along the output rows, as stored
#pragma unroll
      for (int i = 0; i < PPT; ++i) {
        const int e = tid + NT * i, r = e >> 5, cc = e & 31;
        ra[i] = *reinterpret_cast<const u16x8 *>(A + (int64_t)(k0 + r) * lda + m0 + cc * 8);
        rb[i] = *reinterpret_cast<const u16x8 *>(B + (int64_t)(k0 + r) * ldb + n0 + cc * 8);
      }
    }
  };
  auto stash = [&](int buf) {
    bf16_t *as = At + buf * BM * LS, *bs = Bt + buf * BN * LS;   // BM * LS == BK * LT
    if (!TRANS) {
#pragma unroll
      for (int i = 0; i < PPT; ++i) {
        const int e = tid + NT * i, r = e >> 3, cc = e & 7;
        *reinterpret_cast<u16x8 *>(&as[r * LS + cc * 8]) = ra[i];
        *reinterpret_cast<u16x8 *>(&bs[r * LS + cc * 8]) = rb[i];
      }
    } else {        // [k][row] tiles: the transposition happens at the operand reads
#pragma unroll
      for (int i = 0; i < PPT; ++i) {
        const int e = tid + NT * i, r = e >> 5, cc = e & 31;
        *reinterpret_cast<u16x8 *>(&as[r * LT + cc * 8]) = ra[i];
        *reinterpret_cast<u16x8 *>(&bs[r * LT + cc * 8]) = rb[i];
      }
    }
  };

  if (steps > 0) {
    fetch(0);
    stash(0);
  }
  __syncthreads();
  for (int s = 0; s < steps; ++s) {
    const int buf = s & 1;
    const bool more = s + 1 < steps;
    if (more) fetch(s + 1);
    const bf16_t *as = At + buf * BM * LS + (TRANS ? wm : wm * LS);
    const bf16_t *bs = Bt + buf * BN * LS + (TRANS ? wn : wn * LS);
    // Two waves per SIMD: the one in its matrix phase goes ahead of the other's tile traffic (the
    // requests above, the LDS writes below): NT -2 %, TN -3 %.
    __builtin_amdgcn_s_setprio(3);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[4], b[TN];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        a[i] = TRANS ? lds_operand_tr(as + 32 * i, 16 * ks + 8 * h, lane)
                     : *reinterpret_cast<const bf16x8 *>(&as[(32 * i + l32) * LS + 16 * ks + 8 * h]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = TRANS ? lds_operand_tr(bs + 32 * j, 16 * ks + 8 * h, lane)
                     : *reinterpret_cast<const bf16x8 *>(&bs[(32 * j + l32) * LS + 16 * ks + 8 * h]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_s_setprio(0);
    if (more) stash(buf ^ 1);
    __syncthreads();
  }

  // acc[i][j][r]: row wm + 32 i + 8 (r / 4) + 4 h + (r % 4), column wn + 32 j + l32.
  if (OUT_F32) {
    float *C = reinterpret_cast<float *>(Cout) + (int64_t)split * M * ldc;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm + 32 * i + 8 * (r >> 2) + 4 * h + (r & 3);
          C[(int64_t)row * ldc + n0 + wn + 32 * j + l32] = acc[i][j][r];
        }
  } else {
    // bf16 through a wave-private LDS tile of 32 rows x (32 TN) columns: 16-byte row-major
    // stores.  (All waves are past the last barrier of the loop: the operand tiles are free.)
    constexpr int ES = 32 * TN + 8, PPR = 4 * TN;   // tile row stride; 16-byte pieces per row
    bf16_t *C = reinterpret_cast<bf16_t *>(Cout);
    if (colsum) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) v += acc[i][j][r];
        v += __shfl_xor(v, 32, 64);   // the two half-waves hold the two halves of every 8-row group
        if (h == 0) colsum[(int64_t)((m0 + wm) >> 7) * N + n0 + wn + 32 * j + l32] = v;
      }
      if (colmax) {
        static_assert(NW != 8 || 32 * TN == kPooledMaxCols, "one maximum per wave tile of 64 columns");
        float mx = 0.f;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, fabsf(acc[i][j][r]));
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        if (lane == 0) colmax[(int64_t)((m0 + wm) >> 7) * (N / (32 * TN)) + (n0 + wn) / (32 * TN)] = mx;
      }
    }
    bf16_t *tl = reinterpret_cast<bf16_t *>(smem_raw) + wave * (32 * ES);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          tl[(8 * (r >> 2) + 4 * h + (r & 3)) * ES + 32 * j + l32] = to_bf16(acc[i][j][r]);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int u = 0; u < 32 * PPR / 64; ++u) {
        const int e = lane + 64 * u, r = e / PPR, cc = e % PPR;
        const u16x8 piece = *reinterpret_cast<const u16x8 *>(&tl[r * ES + cc * 8]);
        *reinterpret_cast<u16x8 *>(C + (int64_t)(m0 + wm + 32 * i + r) * ldc + n0 + wn + cc * 8) = piece;
      }
    }
  }
}

// out[e] = sum over splits of part[split][e], fixed order.
__global__ void splitk_reduce_kernel(const float *part, int splits, int64_t count, float *out) {
  const int64_t e = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (e >= count) return;
  float4 acc = *reinterpret_cast<const float4 *>(part + e);
  for (int s = 1; s < splits; ++s) {
    const float4 v = *reinterpret_cast<const float4 *>(part + (int64_t)s * count + e);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  *reinterpret_cast<float4 *>(out + e) = acc;
}

// dst [C][R] = src [R][C]^T (bf16), 64 x 64 tiles through LDS.
__global__ void transpose_bf16_kernel(const bf16_t *src, int R, int C, bf16_t *dst) {
  __shared__ bf16_t t[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int e = threadIdx.x; e < 64 * 64; e += blockDim.x) {
    const int r = e >> 6, c = e & 63;
    if (r0 + r < R && c0 + c < C) t[r][c] = src[(int64_t)(r0 + r) * C + c0 + c];
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * 64; e += blockDim.x) {
    const int c = e >> 6, r = e & 63;
    if (r0 + r < R && c0 + c < C) dst[(int64_t)(c0 + c) * R + r0 + r] = t[r][c];
  }
}

constexpr size_t kGemmSmem = (size_t)2 * (BM + BN) * LS * sizeof(bf16_t);
static_assert(BM * LS == BK * LT && BN == BM, "both tile forms share one LDS budget");

template <bool TRANS, bool OUT_F32>
hipError_t launch_gemm(const char *name, const GemmSrc &src, int lda, int ldb, void *C, int ldc, int M, int N,
                       int K, int k_chunk, int splits, hipStream_t st, float *colsum = nullptr,
                       float *colmax = nullptr) {
  constexpr int kGemmWaves = 8;   // two waves per SIMD
  auto kern = &gemm_bf16_kernel<TRANS, OUT_F32, kGemmWaves>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmSmem);
  if (e != hipSuccess) return e;
  const int total = (M / BM) * (N / BN) * splits;
  const int grid = ((total + 7) / 8) * 8;
  WERSA_STAGE(name, st,
              kern<<<grid, 64 * kGemmWaves, kGemmSmem, st>>>(src, lda, ldb, C, ldc, M, N, K, k_chunk, splits, colsum, colmax));
  return hipSuccess;
}

struct BlockPlan {
  int64_t tokens, hidden, act;   // act = tokens * hidden elements
  int splits, k_chunk;           // split of the token axis for the weight gradients
  wersa_desc core;
};

BlockPlan block_plan(const wersa_desc &c) {
  BlockPlan p{};
  p.tokens = (int64_t)c.B * c.n;
  p.hidden = (int64_t)c.H * c.d;
  p.act = p.tokens * p.hidden;
  const int tiles = (int)((p.hidden / BM) * (p.hidden / BN));
  int64_t z = 1024 / tiles;
  if (z > kMaxSplit) z = kMaxSplit;
  if (z > p.tokens / BK) z = p.tokens / BK;
  if (z < 1) z = 1;
  const int64_t steps = (p.tokens / BK + z - 1) / z;
  p.k_chunk = (int)(steps * BK);
  p.splits = (int)((p.tokens + p.k_chunk - 1) / p.k_chunk);
  p.core = c;
  p.core.stride_n = p.hidden;
  p.core.stride_h = c.d;
  p.core.stride_b = (int64_t)c.n * p.hidden;
  return p;
}

// Byte layouts. saved: Q' | K' | V' | A (bf16, (B, n, hidden)) | the core's saved buffer.
struct BlockSaved { size_t qp, kp, vp, a, core, total; };
struct BlockWs { size_t wT[4], qsums, qmax, dA, dQp, dKp, dVp, part, core, total; };
size_t up256(size_t x) { return (x + 255) / 256 * 256; }

BlockSaved block_saved(const BlockPlan &p) {
  BlockSaved s{};
  size_t off = 0;
  const size_t act = up256((size_t)p.act * 2);
  s.qp = off; off += act;
  s.kp = off; off += act;
  s.vp = off; off += act;
  s.a = off;  off += act;
  s.core = off; off += up256(wersa_saved_bytes(&p.core));
  s.total = off;
  return s;
}

BlockWs block_ws(const BlockPlan &p, int bwd) {
  BlockWs w{};
  size_t off = 0;
  if (!bwd) {
    for (int i = 0; i < 4; ++i) { w.wT[i] = off; off += up256((size_t)p.hidden * p.hidden * 2); }
    w.qsums = off; off += up256((size_t)(p.tokens / 128) * p.hidden * 4);   // column sums of Q' per 128 rows
    w.qmax = off;  off += up256((size_t)(p.tokens / 128) * (p.hidden / kPooledMaxCols) * 4);   // and the largest |Q'| per 64 columns
  } else {
    const size_t act = up256((size_t)p.act * 2);
    w.dA = off;  off += act;
    w.dQp = off; off += act;
    w.dKp = off; off += act;
    w.dVp = off; off += act;
    w.part = off; off += up256((size_t)p.splits * p.hidden * p.hidden * 4);
  }
  w.core = off; off += up256(wersa_workspace_bytes(&p.core, bwd));
  w.total = off;
  return w;
}

// The caller's stride fields are ignored (the block lays its tensors out itself): the sizes are
// checked first, then the core descriptor the block builds from them goes through the core's
// own validation.
wersa_status validate_block(const wersa_desc *c) {
  if (!c) return WERSA_ERR_INVALID_ARG;
  if (c->B < 1 || c->H < 1 || c->n < 1 || c->d < 1 || c->m < 1 || c->L < 0) return WERSA_ERR_INVALID_ARG;
  if (c->dtype != WERSA_F32 && c->dtype != WERSA_BF16) return WERSA_ERR_INVALID_ARG;
  if (c->dtype != WERSA_BF16) return WERSA_ERR_UNSUPPORTED;
  const int64_t hidden = (int64_t)c->H * c->d, tokens = (int64_t)c->B * c->n;
  if (hidden % BM != 0 || tokens % BM != 0 || hidden > 16384) return WERSA_ERR_UNSUPPORTED;
  const BlockPlan p = block_plan(*c);
  return validate_desc(&p.core);
}

bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

}  // namespace
}  // namespace wersa

using namespace wersa;

extern "C" {

size_t wersa_block_workspace_bytes(const wersa_desc *desc, int for_backward) {
  if (validate_block(desc) != WERSA_OK) return 0;
  return block_ws(block_plan(*desc), for_backward).total;
}

size_t wersa_block_saved_bytes(const wersa_desc *desc) {
  if (validate_block(desc) != WERSA_OK) return 0;
  return block_saved(block_plan(*desc)).total;
}

int64_t wersa_block_saved_offset(const wersa_desc *desc, int which) {
  if (validate_block(desc) != WERSA_OK) return -1;
  const BlockSaved s = block_saved(block_plan(*desc));
  switch (which) {
    case 0: return (int64_t)s.qp;
    case 1: return (int64_t)s.kp;
    case 2: return (int64_t)s.vp;
    case 3: return (int64_t)s.a;
    case 4: return (int64_t)s.core;
    default: return -1;
  }
}

int64_t wersa_block_workspace_offset(const wersa_desc *desc, int which) {
  if (validate_block(desc) != WERSA_OK) return -1;
  const BlockWs w = block_ws(block_plan(*desc), 1);
  switch (which) {
    case 0: return (int64_t)w.dA;
    case 1: return (int64_t)w.dQp;
    case 2: return (int64_t)w.dKp;
    case 3: return (int64_t)w.dVp;
    default: return -1;
  }
}

wersa_status wersa_block_forward(const wersa_desc *desc, const void *x, const void *wq, const void *wk,
                                 const void *wv, const void *wo, const void *omega_rf,
                                 const float *sigma, const float *gate_w, const float *gate_b,
                                 const float *scale_w, void *y, void *saved, void *workspace,
                                 size_t workspace_bytes, void *hip_stream) {
  const wersa_status vs = validate_block(desc);
  if (vs != WERSA_OK) return vs;
  if (!x || !wq || !wk || !wv || !wo || !omega_rf || !sigma || !gate_w || !gate_b || !scale_w || !y || !saved)
    return WERSA_ERR_INVALID_ARG;
  const BlockPlan p = block_plan(*desc);
  const BlockWs w = block_ws(p, 0);
  const BlockSaved sv = block_saved(p);
  if (!workspace || workspace_bytes < w.total || misaligned(workspace, 256) || misaligned(saved, 256))
    return WERSA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  unsigned char *ws = (unsigned char *)workspace, *sb = (unsigned char *)saved;
  const int hid = (int)p.hidden, M = (int)p.tokens;
  const void *wsrc[4] = {wq, wk, wv, wo};
  bf16_t *wT[4];
  for (int i = 0; i < 4; ++i) {
    wT[i] = (bf16_t *)(ws + w.wT[i]);
    WERSA_STAGE("wersa_transpose", st,
                transpose_bf16_kernel<<<dim3(hid / 64, hid / 64), 256, 0, st>>>((const bf16_t *)wsrc[i], hid, hid, wT[i]));
  }
  bf16_t *proj[3] = {(bf16_t *)(sb + sv.qp), (bf16_t *)(sb + sv.kp), (bf16_t *)(sb + sv.vp)};
  for (int i = 0; i < 3; ++i) {
    GemmSrc src{};
    src.a[0] = (const bf16_t *)x;
    src.b[0] = wT[i];
    src.count = 1;
    if (launch_gemm<false, false>("wersa_gemm_nt", src, hid, hid, proj[i], hid, M, hid, hid, hid, 1, st,
                                  i == 0 ? (float *)(ws + w.qsums) : nullptr,
                                  i == 0 ? (float *)(ws + w.qmax) : nullptr) != hipSuccess)
      return WERSA_ERR_LAUNCH;
  }
  bf16_t *A = (bf16_t *)(sb + sv.a);
  // The pooled query comes out of the W^Q GEMM's epilogue (the core takes it when it can).
  const PooledSums pooled{(const float *)(ws + w.qsums), p.hidden, (const float *)(ws + w.qmax)};
  const wersa_status cs = forward_checked(&p.core, proj[0], proj[1], proj[2], omega_rf, sigma, gate_w, gate_b,
                                          scale_w, A, sb + sv.core, ws + w.core,
                                          wersa_workspace_bytes(&p.core, 0), hip_stream, &pooled);
  if (cs != WERSA_OK) return cs;
  GemmSrc src{};
  src.a[0] = A;
  src.b[0] = wT[3];
  src.count = 1;
  if (launch_gemm<false, false>("wersa_gemm_nt", src, hid, hid, y, hid, M, hid, hid, hid, 1, st) != hipSuccess)
    return WERSA_ERR_LAUNCH;
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

wersa_status wersa_block_backward(const wersa_desc *desc, const void *x, const void *wq, const void *wk,
                                  const void *wv, const void *wo, const void *omega_rf,
                                  const float *sigma, const float *gate_w, const float *gate_b,
                                  const float *scale_w, const void *dy, const void *saved, void *dx,
                                  float *dwq, float *dwk, float *dwv, float *dwo, float *dgate_w,
                                  float *dgate_b, float *dscale_w, float *dsigma, void *workspace,
                                  size_t workspace_bytes, void *hip_stream) {
  const wersa_status vs = validate_block(desc);
  if (vs != WERSA_OK) return vs;
  if (!x || !wq || !wk || !wv || !wo || !omega_rf || !sigma || !gate_w || !gate_b || !scale_w || !dy ||
      !saved || !dx || !dwq || !dwk || !dwv || !dwo)
    return WERSA_ERR_INVALID_ARG;
  const BlockPlan p = block_plan(*desc);
  const BlockWs w = block_ws(p, 1);
  const BlockSaved sv = block_saved(p);
  if (!workspace || workspace_bytes < w.total || misaligned(workspace, 256) || misaligned(saved, 256))
    return WERSA_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  unsigned char *ws = (unsigned char *)workspace;
  const unsigned char *sb = (const unsigned char *)saved;
  const int hid = (int)p.hidden, M = (int)p.tokens;
  const bf16_t *Qp = (const bf16_t *)(sb + sv.qp), *Kp = (const bf16_t *)(sb + sv.kp),
               *Vp = (const bf16_t *)(sb + sv.vp), *A = (const bf16_t *)(sb + sv.a);
  bf16_t *dA = (bf16_t *)(ws + w.dA), *dQp = (bf16_t *)(ws + w.dQp), *dKp = (bf16_t *)(ws + w.dKp),
         *dVp = (bf16_t *)(ws + w.dVp);
  float *part = (float *)(ws + w.part);
  const int64_t wcount = (int64_t)hid * hid;

  auto weight_grad = [&](const bf16_t *left, const bf16_t *right, float *out) -> bool {
    GemmSrc src{};
    src.a[0] = left;
    src.b[0] = right;
    src.count = 1;
    float *target = p.splits == 1 ? out : part;
    if (launch_gemm<true, true>("wersa_gemm_tn", src, hid, hid, target, hid, hid, hid, M, p.k_chunk, p.splits,
                                st) != hipSuccess)
      return false;
    if (p.splits > 1)
      WERSA_STAGE("wersa_splitk_reduce", st,
                  splitk_reduce_kernel<<<(unsigned)((wcount / 4 + 255) / 256), 256, 0, st>>>(part, p.splits, wcount, out));
    return true;
  };

  {  // dA = dY W_out^T: B operand [N = in][K = out] is W_out as stored
    GemmSrc src{};
    src.a[0] = (const bf16_t *)dy;
    src.b[0] = (const bf16_t *)wo;
    src.count = 1;
    if (launch_gemm<false, false>("wersa_gemm_nt", src, hid, hid, dA, hid, M, hid, hid, hid, 1, st) != hipSuccess)
      return WERSA_ERR_LAUNCH;
  }
  if (!weight_grad(A, (const bf16_t *)dy, dwo)) return WERSA_ERR_LAUNCH;
  const wersa_status cs =
      wersa_backward(&p.core, Qp, Kp, Vp, omega_rf, sigma, gate_w, gate_b, scale_w, A, dA, sb + sv.core, dQp, dKp,
                     dVp, dgate_w, dgate_b, dscale_w, dsigma, ws + w.core, wersa_workspace_bytes(&p.core, 1),
                     hip_stream);
  if (cs != WERSA_OK) return cs;
  {  // dX = dQ' W^Q^T + dK' W^K^T + dV' W^V^T
    GemmSrc src{};
    src.a[0] = dQp; src.b[0] = (const bf16_t *)wq;
    src.a[1] = dKp; src.b[1] = (const bf16_t *)wk;
    src.a[2] = dVp; src.b[2] = (const bf16_t *)wv;
    src.count = 3;
    if (launch_gemm<false, false>("wersa_gemm_nt", src, hid, hid, dx, hid, M, hid, hid, hid, 1, st) != hipSuccess)
      return WERSA_ERR_LAUNCH;
  }
  if (!weight_grad((const bf16_t *)x, dQp, dwq)) return WERSA_ERR_LAUNCH;
  if (!weight_grad((const bf16_t *)x, dKp, dwk)) return WERSA_ERR_LAUNCH;
  if (!weight_grad((const bf16_t *)x, dVp, dwv)) return WERSA_ERR_LAUNCH;
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

}  // extern "C"
