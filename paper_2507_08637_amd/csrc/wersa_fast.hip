// MFMA path for bf16 tensors on gfx950 (Section 3.1 steps 3-8 and their derivatives).
//
// Staging (all intermediates that reach HBM are n x d sized; the n x m feature matrices live
// only in registers):
//   haar_stage      X (bf16) -> X_F = W^-1(F (.) W X) as fp16, LDS-staged 64-row tiles
//                   (steps 3, 5, 6 fused; the block-mean form of the gated Haar filter)
//   phiT_contract   sum_t ReLU(X_F Omega)[t,:]^T Y[t,:]  and  sum_t w_t ReLU(X_F Omega)[t,:]
//                   split over n into partials (step 7 + the reductions of step 8;
//                   reused in the backward for dS = Phi_Q^T dN, dz = Phi_Q^T dD)
//   reduce_contract fixed-order sum of the partials, scaled; also bf16 copies as MFMA operands
//   rows            per 64-row block: ReLU(X_F Omega) again, then either the step-8 apply +
//                   normaliser (forward; the same apply form gives dV = Phi_K dS), or
//                   dPhi -> mask -> dX_F -> gated Haar filter of the gradient + per-band
//                   inner products (backward, Q side and K side)
// The projection uses fp16 MFMA operands (X_F in fp16 keeps the sign of X_F Omega right to
// 2^-12, which the ReLU derivative needs); everything downstream of the ReLU uses bf16 MFMA.
#include "wersa_internal.h"

namespace wersa {
namespace {

#include "wersa_small_kernels.inc"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

// MFMA 32x32x16 lane layout (wave64; l32 = lane % 32, h = lane / 32):
//   A operand: row l32, k = 8h + q (q = 0..7)      B operand: column l32, k = 8h + q
//   C/D: acc[i] is row 8*(i/4) + 4h + (i%4), column l32.
__device__ __forceinline__ int acc_row(int i, int h) { return 8 * (i >> 2) + 4 * h + (i & 3); }

__device__ __forceinline__ f32x16 mfma_f16(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// Projection and dPhi chains with their accumulators forced into architectural VGPRs.  In a
// kernel that is given the 512-register budget the compiler keeps every MFMA result in
// accumulation registers, and VALU work on a result then costs one v_accvgpr_read per element;
// the projection (R) and dPhi (G) tiles of the gradient kernel are consumed by VALU at once, so
// they are better off in VGPRs.  The compiler does not see through an asm statement, so each
// statement is hazard-safe on its own: dependent MFMAs are never adjacent (the two chains
// alternate), and the statement ends with the wait states an 8-pass MFMA needs before anything
// (VALU, a copy, a spill) may read its result.
//   chain_first: G = sum_{k<5} ma_k yb_k, R = sum_{k<4} oa_k xb_k.
__device__ __forceinline__ void chain_first(f32x16 &R, f32x16 &G, const f16x8 *oa, const f16x8 *xb,
                                            const bf16x8 *ma, const bf16x8 *yb) {
  asm volatile(
      "v_mfma_f32_32x32x16_bf16 %1, %10, %15, 0\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %2, %6, 0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %11, %16, %1\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %3, %7, %0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %12, %17, %1\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %4, %8, %0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %13, %18, %1\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %5, %9, %0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %14, %19, %1\n\t"
      "s_nop 11"
      : "=&v"(R), "=&v"(G)
      : "v"(oa[0]), "v"(oa[1]), "v"(oa[2]), "v"(oa[3]), "v"(xb[0]), "v"(xb[1]), "v"(xb[2]), "v"(xb[3]),
        "v"(ma[0]), "v"(ma[1]), "v"(ma[2]), "v"(ma[3]), "v"(ma[4]), "v"(yb[0]), "v"(yb[1]), "v"(yb[2]),
        "v"(yb[3]), "v"(yb[4]));
}
// The same chains with their results in fixed registers (tile 0 of a 64-row block: R, G in
// v[192:207], v[208:223]; tile 1: v[224:239], v[240:255]), so that a chain's statement can also
// carry the mask multiplies of the OTHER tile's finished chain, G_i *= clamp(R_i * 2^100, 0, 1),
// written on those registers between its MFMAs: the VALU work runs while the matrix pipe works
// through the chain instead of after it.  Hazards: the masked registers were written by the
// previous chain statement, which ends with the wait states its last MFMA needs; no MFMA here
// reads a register the multiplies write.
__device__ __forceinline__ void chain0_first(f32x16 &R0, f32x16 &G0, const f16x8 *oa, const f16x8 *xb,
                                             const bf16x8 *ma, const bf16x8 *yb) {
  asm volatile(
      "v_mfma_f32_32x32x16_bf16 %1, %10, %15, 0\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %2, %6, 0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %11, %16, %1\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %3, %7, %0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %12, %17, %1\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %4, %8, %0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %13, %18, %1\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %5, %9, %0\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %14, %19, %1\n\t"
      "s_nop 11"
      : "=&{v[192:207]}"(R0), "=&{v[208:223]}"(G0)
      : "v"(oa[0]), "v"(oa[1]), "v"(oa[2]), "v"(oa[3]), "v"(xb[0]), "v"(xb[1]), "v"(xb[2]), "v"(xb[3]),
        "v"(ma[0]), "v"(ma[1]), "v"(ma[2]), "v"(ma[3]), "v"(ma[4]), "v"(yb[0]), "v"(yb[1]), "v"(yb[2]),
        "v"(yb[3]), "v"(yb[4]));
}
// chain of tile 1 (R1, G1) with the mask of tile 0 (G0 *= 1[R0 > 0])
__device__ __forceinline__ void chain1_mask0(f32x16 &R1, f32x16 &G1, f32x16 &G0, const f32x16 &R0,
                                             const f16x8 *oa, const f16x8 *xb, const bf16x8 *ma,
                                             const bf16x8 *yb, float big) {
  float tmp;
  asm volatile(
      "v_mfma_f32_32x32x16_bf16 %1, %12, %17, 0\n\t"
      "v_mul_f32_e64 %3, v192, %23 clamp\n\t"
      "v_mul_f32_e32 v208, v208, %3\n\t"
      "v_mul_f32_e64 %3, v193, %23 clamp\n\t"
      "v_mul_f32_e32 v209, v209, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %4, %8, 0\n\t"
      "v_mul_f32_e64 %3, v194, %23 clamp\n\t"
      "v_mul_f32_e32 v210, v210, %3\n\t"
      "v_mul_f32_e64 %3, v195, %23 clamp\n\t"
      "v_mul_f32_e32 v211, v211, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %13, %18, %1\n\t"
      "v_mul_f32_e64 %3, v196, %23 clamp\n\t"
      "v_mul_f32_e32 v212, v212, %3\n\t"
      "v_mul_f32_e64 %3, v197, %23 clamp\n\t"
      "v_mul_f32_e32 v213, v213, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %5, %9, %0\n\t"
      "v_mul_f32_e64 %3, v198, %23 clamp\n\t"
      "v_mul_f32_e32 v214, v214, %3\n\t"
      "v_mul_f32_e64 %3, v199, %23 clamp\n\t"
      "v_mul_f32_e32 v215, v215, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %14, %19, %1\n\t"
      "v_mul_f32_e64 %3, v200, %23 clamp\n\t"
      "v_mul_f32_e32 v216, v216, %3\n\t"
      "v_mul_f32_e64 %3, v201, %23 clamp\n\t"
      "v_mul_f32_e32 v217, v217, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %6, %10, %0\n\t"
      "v_mul_f32_e64 %3, v202, %23 clamp\n\t"
      "v_mul_f32_e32 v218, v218, %3\n\t"
      "v_mul_f32_e64 %3, v203, %23 clamp\n\t"
      "v_mul_f32_e32 v219, v219, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %15, %20, %1\n\t"
      "v_mul_f32_e64 %3, v204, %23 clamp\n\t"
      "v_mul_f32_e32 v220, v220, %3\n\t"
      "v_mul_f32_e64 %3, v205, %23 clamp\n\t"
      "v_mul_f32_e32 v221, v221, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %7, %11, %0\n\t"
      "v_mul_f32_e64 %3, v206, %23 clamp\n\t"
      "v_mul_f32_e32 v222, v222, %3\n\t"
      "v_mul_f32_e64 %3, v207, %23 clamp\n\t"
      "v_mul_f32_e32 v223, v223, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %16, %21, %1\n\t"
      "s_nop 11"
      : "=&{v[224:239]}"(R1), "=&{v[240:255]}"(G1), "+{v[208:223]}"(G0), "=&v"(tmp)
      : "v"(oa[0]), "v"(oa[1]), "v"(oa[2]), "v"(oa[3]), "v"(xb[0]), "v"(xb[1]), "v"(xb[2]), "v"(xb[3]),
        "v"(ma[0]), "v"(ma[1]), "v"(ma[2]), "v"(ma[3]), "v"(ma[4]), "v"(yb[0]), "v"(yb[1]), "v"(yb[2]),
        "v"(yb[3]), "v"(yb[4]), "{v[192:207]}"(R0), "s"(big));
}
// chain of tile 0 (R0, G0) of the next feature tile with the mask of tile 1 (G1 *= 1[R1 > 0])
__device__ __forceinline__ void chain0_mask1(f32x16 &R0, f32x16 &G0, f32x16 &G1, const f32x16 &R1,
                                             const f16x8 *oa, const f16x8 *xb, const bf16x8 *ma,
                                             const bf16x8 *yb, float big) {
  float tmp;
  asm volatile(
      "v_mfma_f32_32x32x16_bf16 %1, %12, %17, 0\n\t"
      "v_mul_f32_e64 %3, v224, %23 clamp\n\t"
      "v_mul_f32_e32 v240, v240, %3\n\t"
      "v_mul_f32_e64 %3, v225, %23 clamp\n\t"
      "v_mul_f32_e32 v241, v241, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %4, %8, 0\n\t"
      "v_mul_f32_e64 %3, v226, %23 clamp\n\t"
      "v_mul_f32_e32 v242, v242, %3\n\t"
      "v_mul_f32_e64 %3, v227, %23 clamp\n\t"
      "v_mul_f32_e32 v243, v243, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %13, %18, %1\n\t"
      "v_mul_f32_e64 %3, v228, %23 clamp\n\t"
      "v_mul_f32_e32 v244, v244, %3\n\t"
      "v_mul_f32_e64 %3, v229, %23 clamp\n\t"
      "v_mul_f32_e32 v245, v245, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %5, %9, %0\n\t"
      "v_mul_f32_e64 %3, v230, %23 clamp\n\t"
      "v_mul_f32_e32 v246, v246, %3\n\t"
      "v_mul_f32_e64 %3, v231, %23 clamp\n\t"
      "v_mul_f32_e32 v247, v247, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %14, %19, %1\n\t"
      "v_mul_f32_e64 %3, v232, %23 clamp\n\t"
      "v_mul_f32_e32 v248, v248, %3\n\t"
      "v_mul_f32_e64 %3, v233, %23 clamp\n\t"
      "v_mul_f32_e32 v249, v249, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %6, %10, %0\n\t"
      "v_mul_f32_e64 %3, v234, %23 clamp\n\t"
      "v_mul_f32_e32 v250, v250, %3\n\t"
      "v_mul_f32_e64 %3, v235, %23 clamp\n\t"
      "v_mul_f32_e32 v251, v251, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %15, %20, %1\n\t"
      "v_mul_f32_e64 %3, v236, %23 clamp\n\t"
      "v_mul_f32_e32 v252, v252, %3\n\t"
      "v_mul_f32_e64 %3, v237, %23 clamp\n\t"
      "v_mul_f32_e32 v253, v253, %3\n\t"
      "v_mfma_f32_32x32x16_f16 %0, %7, %11, %0\n\t"
      "v_mul_f32_e64 %3, v238, %23 clamp\n\t"
      "v_mul_f32_e32 v254, v254, %3\n\t"
      "v_mul_f32_e64 %3, v239, %23 clamp\n\t"
      "v_mul_f32_e32 v255, v255, %3\n\t"
      "v_mfma_f32_32x32x16_bf16 %1, %16, %21, %1\n\t"
      "s_nop 11"
      : "=&{v[192:207]}"(R0), "=&{v[208:223]}"(G0), "+{v[240:255]}"(G1), "=&v"(tmp)
      : "v"(oa[0]), "v"(oa[1]), "v"(oa[2]), "v"(oa[3]), "v"(xb[0]), "v"(xb[1]), "v"(xb[2]), "v"(xb[3]),
        "v"(ma[0]), "v"(ma[1]), "v"(ma[2]), "v"(ma[3]), "v"(ma[4]), "v"(yb[0]), "v"(yb[1]), "v"(yb[2]),
        "v"(yb[3]), "v"(yb[4]), "{v[224:239]}"(R1), "s"(big));
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}
// x[lane] + x[lane ^ 32] in every lane: one swap of the upper half of a register with the lower
// half of its copy (a VALU instruction of gfx950) and an add, instead of an exchange through LDS.
__device__ __forceinline__ float xor32_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float wave_sum64(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Pack accumulator registers 8a .. 8a+7 into one bf16 MFMA operand. With this choice k-slot
// (h, q) of the consuming MFMA stands for accumulator row 16a + 8*(q/4) + 4h + (q%4); the other
// operand must be fetched in the same order (two runs of four consecutive indices).
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8 pack_half(const f32x16 &v, int a) {
  bf16x8 p;
#pragma unroll
  for (int j = 0; j < 4; ++j) {   // one packed conversion per pair
    f32x2 f;
    f[0] = v[8 * a + 2 * j];
    f[1] = v[8 * a + 2 * j + 1];
    const bf16x2_t c = __builtin_convertvector(f, bf16x2_t);
    p[2 * j] = c[0];
    p[2 * j + 1] = c[1];
  }
  return p;
}
// The matching operand: indices base + 4h + {0..3} and base + 8 + 4h + {0..3} of a row in LDS.
__device__ __forceinline__ bf16x8 lds_perm8(const bf16_t *row, int base, int h) {
  const bf16x4 lo = *reinterpret_cast<const bf16x4 *>(row + base + 4 * h);
  const bf16x4 hi = *reinterpret_cast<const bf16x4 *>(row + base + 8 + 4 * h);
  bf16x8 r;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    r[q] = lo[q];
    r[4 + q] = hi[q];
  }
  return r;
}

// Sum over the 32 lanes of a half-wave, result in every lane: two quad exchanges and two row
// rotations inside each group of 16 lanes (DPP), then one swap of the two groups (swizzle).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float half_wave_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x124>(v);   // row_ror 4
  v += dpp_move<0x128>(v);   // row_ror 8
  v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));   // lane ^ 16
  return v;
}

// ------------------------------------------------------------------------------------
// Per-call constants: block 0 writes the scalars; every block transposes its share of Omega
// into Omega^T in fp16 ([m][d]), the projection's MFMA operand.  (The filter coefficients of
// the block-mean form come from the gate kernel.)
// ------------------------------------------------------------------------------------
struct SetupArgs {
  const float *sigma;
  float bw_floor;
  const bf16_t *omega;
  int d, m, matrices;
  float *scalars;
  _Float16 *omT;
  int blocks;   // workgroups of 256 threads that cover matrices * d * m elements (0: nothing to do)
};
inline int setup_blocks(int d, int m, int matrices) { return (matrices * d * m + 255) / 256; }
__device__ __forceinline__ void setup_body(const SetupArgs &a, int block) {
  if (block == 0 && threadIdx.x == 0) {
    const float s = *a.sigma;
    const float se = fmaxf(s, a.bw_floor);
    a.scalars[0] = 1.0f / (se * sqrtf((float)a.m));
    a.scalars[1] = se;
    a.scalars[2] = s > a.bw_floor ? 1.0f : 0.0f;
    a.scalars[3] = 1.0f;
  }
  const int e = block * 256 + threadIdx.x;
  if (e < a.matrices * a.d * a.m) {   // one or two d x m matrices, each transposed on its own
    const int mat = e / (a.d * a.m), w = e % (a.d * a.m);
    const int r = w / a.d, j = w % a.d;
    a.omT[e] = (_Float16)bf16_to_f32(a.omega[(int64_t)mat * a.d * a.m + (int64_t)j * a.m + r]);
  }
}
__global__ __launch_bounds__(256) void setup_kernel(SetupArgs a) { setup_body(a, blockIdx.x); }

// ------------------------------------------------------------------------------------
// Column sums of Q for the pooled query: 16-byte loads, one partial per (slice, chunk).
// Grid (chunks + su.blocks, slices): the workgroups past `chunks` of slice 0 carry the per-call
// constants (one launch fewer at the head of the forward pass); those of the other slices exit.
// ------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void qbar_partial_kernel(const bf16_t *q, View v, int n,
                                                          int rows_per_chunk, float *part, int chunks,
                                                          SetupArgs su, float *amax_part) {
  constexpr int CPR = DH / 8;        // 16-byte chunks per row
  constexpr int RPI = 256 / CPR;     // rows per iteration
  if ((int)blockIdx.x >= chunks) {
    if (blockIdx.y == 0) setup_body(su, blockIdx.x - chunks);
    return;
  }
  const int slice = blockIdx.y, chunk = blockIdx.x;
  const int t0 = chunk * rows_per_chunk, t1 = min(n, t0 + rows_per_chunk);
  const int cc = threadIdx.x % CPR, rr = threadIdx.x / CPR;
  const bf16_t *qs = q + v.slice_base(slice) + cc * 8;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  // largest magnitude seen: integer maximum of the values with their sign bits cleared (packed 16-bit)
  u16x8 mx = {0, 0, 0, 0, 0, 0, 0, 0};
  const u16x8 magn = {0x7fff, 0x7fff, 0x7fff, 0x7fff, 0x7fff, 0x7fff, 0x7fff, 0x7fff};
  auto track = [&](const u16x8 &x) { mx = __builtin_elementwise_max(mx, x & magn); };
  int t = t0 + rr;
  for (; t + 7 * RPI < t1; t += 8 * RPI) {   // eight independent loads in flight
    u16x8 x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = *reinterpret_cast<const u16x8 *>(qs + (int64_t)(t + u * RPI) * v.sn);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      track(x[u]);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += bf16_to_f32(x[u][e]);
    }
  }
  for (; t < t1; t += RPI) {
    const u16x8 x = *reinterpret_cast<const u16x8 *>(qs + (int64_t)t * v.sn);
    track(x);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += bf16_to_f32(x[e]);
  }
  __shared__ float red[RPI][DH + 1];
  __shared__ float amax_w[4];
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rr][cc * 8 + e] = acc[e];
  if (amax_part) {   // (NaN and infinity compare as the largest magnitudes and are passed on as such)
    unsigned short m16 = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) m16 = mx[e] > m16 ? mx[e] : m16;
    float m = bf16_to_f32(m16);
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if ((threadIdx.x & 63) == 0) amax_w[threadIdx.x >> 6] = m;
  }
  __syncthreads();
  if (threadIdx.x < DH) {
    float s = 0.f;
    for (int r = 0; r < RPI; ++r) s += red[r][threadIdx.x];
    part[((int64_t)slice * chunks + chunk) * DH + threadIdx.x] = s;
  }
  if (amax_part && threadIdx.x == 0)
    amax_part[(int64_t)slice * chunks + chunk] = fmaxf(fmaxf(amax_w[0], amax_w[1]), fmaxf(amax_w[2], amax_w[3]));
}

// ------------------------------------------------------------------------------------
// Gated Haar filter in block-mean form on one column, RS consecutive rows held by a thread.
//   bs_l = sum over the aligned 2^l block;  out = sum_l coef_l * bs_l
// `upper` is sum_{l > log2 RS} coef_l * bs_l for the blocks that contain this segment.
// ------------------------------------------------------------------------------------
template <int RS>
__device__ __forceinline__ void filter_segment(float (&v)[RS], const float *coef, float upper) {
  constexpr int LV = RS == 32 ? 5 : 4;
  static_assert(RS == 16 || RS == 32, "segment of 16 or 32 rows");
  float bs[LV + 1][RS];
#pragma unroll
  for (int i = 0; i < RS; ++i) bs[0][i] = v[i];
#pragma unroll
  for (int l = 1; l <= LV; ++l)
#pragma unroll
    for (int k = 0; k < (RS >> l); ++k) bs[l][k] = bs[l - 1][2 * k] + bs[l - 1][2 * k + 1];
  float T[LV + 1][RS];
  T[LV][0] = fmaf(coef[LV], bs[LV][0], upper);
#pragma unroll
  for (int l = LV - 1; l >= 0; --l)
#pragma unroll
    for (int k = 0; k < (RS >> l); ++k) T[l][k] = fmaf(coef[l], bs[l][k], T[l + 1][k >> 1]);
#pragma unroll
  for (int i = 0; i < RS; ++i) v[i] = T[0][i];
}
template <int RS>
__device__ __forceinline__ float segment_sum(const float (&v)[RS]) {
  float s[RS];
#pragma unroll
  for (int i = 0; i < RS; ++i) s[i] = v[i];
#pragma unroll
  for (int w = RS / 2; w >= 1; w >>= 1)
#pragma unroll
    for (int k = 0; k < w; ++k) s[k] = s[2 * k] + s[2 * k + 1];
  return s[0];
}

// X (bf16, strided) -> X_F (fp16, contiguous [slices][n][DH]); one 64-row tile per workgroup.
// Steps: coalesced 16-byte loads into LDS; one thread per (column, row segment) computes the
// nested block sums (in registers up to the segment, through LDS above it) and the filtered
// values; fp16 results go back to LDS and leave with coalesced 16-byte stores.
// tile_add (L > 6, else nullptr): [slices][ceil(n / 64)][DH], the per-tile addend of the levels above 6.
template <int DH>
__global__ __launch_bounds__(256) void haar_stage_kernel(const bf16_t *x, View v, int n,
                                                        const float *coef, const float *tile_add, _Float16 *xf) {
  constexpr int SEGS = 256 / DH;   // row segments per column: 4 (DH=64) or 2 (DH=128)
  constexpr int RS = 64 / SEGS;    // rows per segment: 16 or 32
  constexpr int CPR = DH / 8;
  __shared__ __attribute__((aligned(16))) bf16_t tile[64 * DH];
  __shared__ float segsum[SEGS][DH];
  __shared__ float cf[8];
  const int slice = blockIdx.y, t0 = blockIdx.x * 64;
  const int tid = threadIdx.x;
  if (tid < 8) cf[tid] = coef[slice * kCoefStride + tid];
  const bf16_t *xs = x + v.slice_base(slice);
  for (int e = tid; e < 64 * CPR; e += 256) {
    const int r = e / CPR, cc = e % CPR;
    u16x8 val;
    if (t0 + r < n) val = *reinterpret_cast<const u16x8 *>(xs + (int64_t)(t0 + r) * v.sn + cc * 8);
    else
#pragma unroll
      for (int q = 0; q < 8; ++q) val[q] = 0;
    *reinterpret_cast<u16x8 *>(&tile[r * DH + cc * 8]) = val;
  }
  __syncthreads();
  const int c = tid % DH, seg = tid / DH;
  float vals[RS];
#pragma unroll
  for (int i = 0; i < RS; ++i) vals[i] = bf16_to_f32(tile[(seg * RS + i) * DH + c]);
  segsum[seg][c] = segment_sum<RS>(vals);
  __syncthreads();
  float upper;
  if (SEGS == 4) {
    const float s5 = segsum[seg & ~1][c] + segsum[seg | 1][c];
    const float s6 = (segsum[0][c] + segsum[1][c]) + (segsum[2][c] + segsum[3][c]);
    upper = fmaf(cf[5], s5, cf[6] * s6);
  } else {
    upper = cf[6] * (segsum[0][c] + segsum[1][c]);
  }
  if (tile_add) upper += tile_add[((int64_t)slice * gridDim.x + blockIdx.x) * DH + c];
  filter_segment<RS>(vals, cf, upper);
  _Float16 *tile16 = reinterpret_cast<_Float16 *>(tile);
#pragma unroll
  for (int i = 0; i < RS; ++i) tile16[(seg * RS + i) * DH + c] = (_Float16)vals[i];
  __syncthreads();
  _Float16 *out = xf + ((int64_t)slice * n + t0) * DH;
  for (int e = tid; e < 64 * CPR; e += 256) {
    const int r = e / CPR, cc = e % CPR;
    if (t0 + r < n)
      *reinterpret_cast<u16x8 *>(out + (int64_t)r * DH + cc * 8) =
          *reinterpret_cast<const u16x8 *>(&tile[r * DH + cc * 8]);
  }
}

// float32 -> bf16 storage with the hardware conversion (round to nearest even)
__device__ __forceinline__ bf16_t cvt_bf16(float f) {
  return __builtin_bit_cast(bf16_t, (__bf16)f);
}

// The gated Haar filter as a stage of its own on bf16 tensors (steps 3, 5, 6 of Section 3.1; the
// stage entry point): X -> X_F in the same layout and dtype, up to six levels, one tile of 64 rows x
// 64 columns per workgroup.  Rows move in 16-byte pieces both ways; the filter is evaluated in
// block-mean form, one thread per (column, 16-row segment), the 32- and 64-row sums through LDS;
// no float copy of the tile exists anywhere.  filt: [slices][L + 1] (band order of Algorithm 2).
__global__ __launch_bounds__(256) void haar_filter_bf16_kernel(const bf16_t *x, bf16_t *y, View v, int n, int d,
                                                              const float *filt, int L) {
  constexpr int TC = 64, RS = 16, CPR = TC / 8;
  __shared__ __attribute__((aligned(16))) bf16_t tile[64 * TC];
  __shared__ float segsum[4][TC];
  __shared__ float cf[8];
  const int slice = blockIdx.z, t0 = blockIdx.x * 64, c0 = blockIdx.y * TC;
  const int tid = threadIdx.x;
  if (tid < 8) {   // block-mean coefficients: coef_0 = F_0, coef_l = (F_l - F_{l-1}) / 2^l, 0 above L
    const float *F = filt + (int64_t)slice * (L + 1);
    cf[tid] = tid == 0 ? F[0] : (tid <= L ? (F[tid] - F[tid - 1]) / (float)(1 << tid) : 0.f);
  }
  const int64_t base = v.slice_base(slice);
  u16x8 piece[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int e = tid + 256 * u, r = e / CPR, cc = e % CPR;
    const bool ok = t0 + r < n && c0 + cc * 8 < d;
    // (rows past n and columns past d read as zeros: Algorithm 2's padding)
    piece[u] = *reinterpret_cast<const u16x8 *>(x + base + (int64_t)(ok ? t0 + r : 0) * v.sn + (ok ? c0 + cc * 8 : 0));
    if (!ok)
#pragma unroll
      for (int q = 0; q < 8; ++q) piece[u][q] = 0;
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int e = tid + 256 * u;
    *reinterpret_cast<u16x8 *>(&tile[(e / CPR) * TC + (e % CPR) * 8]) = piece[u];
  }
  __syncthreads();
  const int c = tid % TC, seg = tid / TC;
  float vals[RS];
#pragma unroll
  for (int i = 0; i < RS; ++i) vals[i] = bf16_to_f32(tile[(seg * RS + i) * TC + c]);
  segsum[seg][c] = segment_sum<RS>(vals);
  __syncthreads();
  const float s5 = segsum[seg & ~1][c] + segsum[seg | 1][c];
  const float s6 = (segsum[0][c] + segsum[1][c]) + (segsum[2][c] + segsum[3][c]);
  filter_segment<RS>(vals, cf, fmaf(cf[5], s5, cf[6] * s6));
#pragma unroll
  for (int i = 0; i < RS; ++i) tile[(seg * RS + i) * TC + c] = cvt_bf16(vals[i]);
  __syncthreads();
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int e = tid + 256 * u, r = e / CPR, cc = e % CPR;
    if (t0 + r < n && c0 + cc * 8 < d)
      *reinterpret_cast<u16x8 *>(y + base + (int64_t)(t0 + r) * v.sn + c0 + cc * 8) =
          *reinterpret_cast<const u16x8 *>(&tile[r * TC + cc * 8]);
  }
}

// ------------------------------------------------------------------------------------
// Small helpers for the chained MFMAs.
// ------------------------------------------------------------------------------------
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// ReLU on a packed bf16 operand: as 16-bit integers, negative floats are negative integers.
__device__ __forceinline__ bf16x8 relu_bf16x8(bf16x8 p) {
  s16x8 s = __builtin_bit_cast(s16x8, p);
  const s16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  s = __builtin_elementwise_max(s, zero);
  return __builtin_bit_cast(bf16x8, s);
}
// acc + sum_q p[q] * w[q] with bf16 pair dot products (float32 accumulate)
__device__ __forceinline__ float dot8_bf16(bf16x8 p, bf16x8 w, float acc) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    bf16x2 a, b;
    a[0] = p[2 * j]; a[1] = p[2 * j + 1];
    b[0] = w[2 * j]; b[1] = w[2 * j + 1];
    acc = __builtin_amdgcn_fdot2_f32_bf16(a, b, acc, false);
  }
  return acc;
}
__device__ __forceinline__ bf16x8 splat_bf16x8(float v) {
  bf16x8 r;
#pragma unroll
  for (int q = 0; q < 8; ++q) r[q] = (__bf16)v;
  return r;
}

// Transposing LDS read of gfx950 (ds_read_b64_tr_b16): within each group of 16 lanes, lane i
// passes the address of four consecutive 16-bit values, taken as row i / 4, columns
// 4 (i % 4) .. + 3 of a 4 x 16 block, and receives column i of that block.  (Lane mapping
// checked on the GPU with an index-valued LDS array.)
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x4 lds_read_tr4(const bf16_t *p) {
  typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
  return __builtin_bit_cast(bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p));
}

// The same packing as pack_half into an fp16 operand.
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f16x8 pack_half_f16(const f32x16 &v, int a) {
  f16x8 p;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f32x2 f;
    f[0] = v[8 * a + 2 * j];
    f[1] = v[8 * a + 2 * j + 1];
    const f16x2_t c = __builtin_convertvector(f, f16x2_t);
    p[2 * j] = c[0];
    p[2 * j + 1] = c[1];
  }
  return p;
}

// In-kernel stage A (head dimension 64): the gated Haar filter of one aligned 64-row block is
// the product with a 64 x 64 matrix G (from the block-mean coefficients of the slice), so the kernels
// that consume X_F take the raw rows of Q or K and form X_F^T = X^T G^T on the matrix cores.
// G[t'][t] depends only on the highest bit in which t' and t differ: g_k = sum of coef_l over
// l >= k, k = 0 for t' == t, else (position of that bit) + 1.  For the matrix cores G is split
// into a bf16 high part and a bf16 low part (the gradients are sensitive to a relative error of
// 2^-9 in the filter), and its B operands (column t', k-slot t = 8 j + q) come out of a small
// table T[part][t' % 8][(t' / 8) ^ j][q] = part of g at t' ^ t, one 16-byte read each.
__device__ __forceinline__ void build_filter_table(bf16_t *T, const float *coef8, int tid, int nthreads) {
  float g[7], acc = 0.f;
#pragma unroll
  for (int l = 6; l >= 0; --l) {
    acc += coef8[l];
    g[l] = acc;
  }
  for (int e = tid; e < 512; e += nthreads) {
    const int b = e >> 6, xh = (e >> 3) & 7, q = e & 7;
    const int x = 8 * xh + (b ^ q);
    const int lvl = x ? 32 - __clz(x) : 0;
    float v = g[0];
#pragma unroll
    for (int k = 1; k < 7; ++k) v = (lvl == k) ? g[k] : v;
    const __bf16 hi = (__bf16)v;
    const __bf16 lo = (__bf16)(v - (float)hi);
    T[e] = __builtin_bit_cast(bf16_t, hi);
    T[512 + e] = __builtin_bit_cast(bf16_t, lo);
  }
}
__device__ __forceinline__ bf16x8 filter_operand(const bf16_t *T, int part, int trow, int j) {
  return *reinterpret_cast<const bf16x8 *>(&T[part * 512 + (((trow & 7) << 3) | ((trow >> 3) ^ j)) * 8]);
}
// This is the A operand of that product from a row-major bf16 tile [t][stride]: operand row
// lane % 32 is tile column col0 + lane % 32 (PERM: with bits 2 and 3 of lane % 32 swapped),
// k-slot (h, q) is tile row 16 ks + 8 h + q.  With PERM, pack_half of the result delivers the
// columns in natural order (k-slot (h, q) of half a is column 16 a + 8 h + q).
template <bool PERM>
__device__ __forceinline__ bf16x8 tile_cols_operand(const bf16_t *tile, int stride, int col0, int ks, int lane) {
  const int i16 = lane & 15, g16 = lane >> 4;
  int k = i16 & 3;
  if (PERM) k = ((k & 1) << 1) | (k >> 1);
  const bf16_t *p = tile + (16 * ks + 8 * (g16 >> 1) + (i16 >> 2)) * stride + col0 + 16 * (g16 & 1) + 4 * k;
  const bf16x4 lo = lds_read_tr4(p), hi = lds_read_tr4(p + 4 * stride);
  bf16x8 r;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    r[q] = lo[q];
    r[4 + q] = hi[q];
  }
  return r;
}

// ------------------------------------------------------------------------------------
// phiT_contract: for the rows of one chunk and the features [f0, f0 + 4*FW) of one slice
//   Spart[r][c] = sum_t ReLU(X_F Omega)[t][r] * (Y[t][c] / rowdiv_t)
//   zpart[r]    = sum_t w_t * ReLU(X_F Omega)[t][r]
// Four waves split the features; each wave keeps its Omega operands in registers and chains
// the projection's accumulators (rows t on registers) straight into the second MFMA as the
// A operand.  X_F and Y tiles of 64 rows go through double-buffered LDS (Y transposed so that
// t runs along the operand's k index); the next tile is fetched while the current one is used.
// ------------------------------------------------------------------------------------
// PREP (backward, Q side): Y = dO, rowdiv = D, and the weights are computed here instead of
// read: w_t = dD_t = -<dO_t, O_t> / D_t from the rows of O (`orows`, laid out like Y).  The
// feature block 0 also writes dD [slices][n] for the gradient rows kernel and one partial sum
// of dD per (slice, chunk) for d sigma.
// Head dimension 64 (FUSE): `xf` is not read; the rows of X (Q or K, bf16, view vx) are staged
// raw and each step starts with X_F = G X for its tile, one 32 x 32 quarter per wave, written
// to LDS in fp16 for the projection.
// RAGGED: n % 64 != 0, rows past n count as zeros with weight 0.  DEEP: L > 6, the filter's levels
// above 6 enter as the per-tile addend tile_add [slices][ceil(n / 64)][DH] (the accumulators of X_F start there).
template <int DH, int FW, bool PREP, bool RAGGED, bool DEEP>
__global__ __launch_bounds__(256, 2) void phiT_contract_kernel(
    const _Float16 *xf, const bf16_t *xraw, View vx, const float *coef, const float *tile_add,
    const bf16_t *y, View vy, const float *rowdiv, const float *w,
    const bf16_t *orows, float *dDout, float *dDpart,
    const _Float16 *omT, int n, int m, int rows_per_chunk, float *Spart, float *zpart) {
  constexpr bool FUSE = (DH == 64);
  constexpr int KS = DH / 16;   // k-steps of the projection
  constexpr int RT = FW / 32;   // feature tiles per wave
  constexpr int CT = DH / 32;   // column tiles of Y
  constexpr int CPR = DH / 8;   // 16-byte pieces per row
  constexpr int LPT = 64 * CPR / 256;   // pieces per thread per tile
  constexpr int YS = DH + 32;   // row stride (elements) of the Y tile [t][column]: 64 bytes past a multiple
                                // of 256, so the four rows of a transposing read fall into different bank quarters
  constexpr int XS = DH + 8;    // row stride (elements) of the X_F tile
  __shared__ __attribute__((aligned(16))) bf16_t yt[2][64 * YS];
  __shared__ __attribute__((aligned(16))) _Float16 xt[2][64 * XS];   // FUSE: raw bf16 rows of X
  __shared__ __attribute__((aligned(16))) _Float16 xq[FUSE ? 64 * XS : 8];   // FUSE: X_F of the current tile
  __shared__ __attribute__((aligned(16))) bf16_t gt[FUSE ? 1024 : 8];        // FUSE: filter operand table
  __shared__ __attribute__((aligned(16))) bf16_t wl[2][64];
  const int slice = blockIdx.z, chunk = blockIdx.x, chunks = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int f0 = blockIdx.y * (4 * FW) + wave * FW;
  const int t_begin = chunk * rows_per_chunk, t_end = min(n, t_begin + rows_per_chunk);
  const int steps = (t_end - t_begin + 63) / 64;   // the last tile of the sequence may be partial

  // Omega^T operands of this wave's features: B operand, column = feature, k = 8h + q.
  f16x8 om[RT][KS];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      om[rt][ks] = *reinterpret_cast<const f16x8 *>(omT + (int64_t)(f0 + 32 * rt + l32) * DH + 16 * ks + 8 * h);

  f32x16 S[RT][CT];
  float zacc[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    zacc[rt] = 0.f;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) S[rt][ct] = zero16();
  }
  const _Float16 *xs = FUSE ? nullptr : xf + (int64_t)slice * n * DH;
  const bf16_t *xrs = FUSE ? xraw + vx.slice_base(slice) : nullptr;
  const bf16_t *ys = y + vy.slice_base(slice);
  const float *rd = rowdiv ? rowdiv + (int64_t)slice * n : nullptr;
  if (FUSE) build_filter_table(gt, coef + slice * kCoefStride, tid, 256);   // visible after the first barrier below
  const float *ws = w ? w + (int64_t)slice * n : nullptr;

  // X_F and Y pieces are taken row-major (coalesced) and stored as they are; the Y operand
  // (t along k) comes out of its tile through transposing LDS reads.
  u16x8 yr[LPT], xr[LPT];
  float inv[LPT], wv = 1.0f;
  // PREP: the rows of O come in like those of Y (the thread that holds piece cc of row r of dO
  // holds the same piece of O); the CPR partial dot products of a row sit in neighbouring lanes.
  u16x8 orw[PREP ? LPT : 1];
  float dsum = 0.f;
  const bf16_t *os = PREP ? orows + vy.slice_base(slice) : nullptr;
  // RAGGED: rows past n (partial last tile) count as zeros with weight 0: the address is clamped
  // to the last row and the value replaced.
  // Whole tiles (the plain instances): one running pointer per tensor, advanced by a tile per
  // call (the tiles are requested in order); piece i sits i * (256 / CPR) rows further on.
  constexpr int RPP = 256 / CPR;   // rows between a thread's pieces
  const int r0 = tid / CPR, c0 = (tid % CPR) * 8;
  const int64_t xsn = FUSE ? vx.sn : DH;
  const u16x8 *px = reinterpret_cast<const u16x8 *>((FUSE ? xrs : reinterpret_cast<const bf16_t *>(xs)) +
                                                    (int64_t)(t_begin + r0) * xsn + c0);
  const u16x8 *py = reinterpret_cast<const u16x8 *>(ys + (int64_t)(t_begin + r0) * vy.sn + c0);
  const u16x8 *po = PREP ? reinterpret_cast<const u16x8 *>(os + (int64_t)(t_begin + r0) * vy.sn + c0) : nullptr;
  const float *prd = rd ? rd + t_begin + r0 : nullptr;
  const float *pws = ws ? ws + t_begin + tid : nullptr;
  auto fetch = [&](int t0) {
    if (!RAGGED) {
#pragma unroll
      for (int i = 0; i < LPT; ++i) {
        xr[i] = *reinterpret_cast<const u16x8 *>(reinterpret_cast<const bf16_t *>(px) + i * RPP * xsn);
        yr[i] = *reinterpret_cast<const u16x8 *>(reinterpret_cast<const bf16_t *>(py) + i * RPP * vy.sn);
        if (PREP) orw[i] = *reinterpret_cast<const u16x8 *>(reinterpret_cast<const bf16_t *>(po) + i * RPP * vy.sn);
        inv[i] = prd ? prd[i * RPP] : 1.0f;   // divided at the stash, when the load has landed
      }
      if (!PREP && tid < 64) wv = pws ? *pws : 1.0f;
      px = reinterpret_cast<const u16x8 *>(reinterpret_cast<const bf16_t *>(px) + 64 * xsn);
      py = reinterpret_cast<const u16x8 *>(reinterpret_cast<const bf16_t *>(py) + 64 * vy.sn);
      if (PREP) po = reinterpret_cast<const u16x8 *>(reinterpret_cast<const bf16_t *>(po) + 64 * vy.sn);
      if (prd) prd += 64;
      if (pws) pws += 64;
      return;
    }
    const int last = RAGGED ? n - t0 - 1 : 63;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int e = tid + 256 * i, r = e / CPR, cc = e % CPR;
      const bool bad = RAGGED && r > last;
      const int rc = t0 + (RAGGED ? min(r, last) : r);
      xr[i] = FUSE ? *reinterpret_cast<const u16x8 *>(xrs + (int64_t)rc * vx.sn + cc * 8)
                   : *reinterpret_cast<const u16x8 *>(xs + (int64_t)rc * DH + cc * 8);
      yr[i] = *reinterpret_cast<const u16x8 *>(ys + (int64_t)rc * vy.sn + cc * 8);
      if (PREP) orw[i] = *reinterpret_cast<const u16x8 *>(os + (int64_t)rc * vy.sn + cc * 8);
      inv[i] = rd ? rd[rc] : 1.0f;   // divided at the stash, when the load has landed
      if (bad) {
#pragma unroll
        for (int q = 0; q < 8; ++q) { xr[i][q] = 0; yr[i][q] = 0; }
        inv[i] = 1.0f;
      }
    }
    if (!PREP && tid < 64) wv = (RAGGED && tid > last) ? 0.f : (ws ? ws[t0 + tid] : 1.0f);
  };
  int t_stash = t_begin;   // first row of the tile the registers hold
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int e = tid + 256 * i, r = e / CPR, cc = e % CPR;
      *reinterpret_cast<u16x8 *>(&xt[buf][r * XS + cc * 8]) = xr[i];
      if (rd) {
        const float rinv = 1.0f / inv[i];
        u16x8 sc;
#pragma unroll
        for (int q = 0; q < 8; ++q) sc[q] = cvt_bf16(bf16_to_f32(yr[i][q]) * rinv);
        *reinterpret_cast<u16x8 *>(&yt[buf][r * YS + cc * 8]) = sc;
      } else {
        *reinterpret_cast<u16x8 *>(&yt[buf][r * YS + cc * 8]) = yr[i];
      }
    }
    if (PREP) {
      static_assert(!PREP || CPR == 8 || CPR == 16, "row pieces sit in 8 or 16 neighbouring lanes");
#pragma unroll
      for (int i = 0; i < LPT; ++i) {
        const int e = tid + 256 * i, r = e / CPR, cc = e % CPR;
        // (rows past n hold zeros in yr and 1 in inv: their dD is 0)
        float dot = dot8_bf16(__builtin_bit_cast(bf16x8, orw[i]), __builtin_bit_cast(bf16x8, yr[i]), 0.f);
        dot += dpp_move<0xB1>(dot);    // lane ^ 1
        dot += dpp_move<0x4E>(dot);    // lane ^ 2
        dot += dpp_move<0x141>(dot);   // mirror inside each group of 8 lanes: the other quad's sum
        if (CPR == 16) dot += dpp_move<0x140>(dot);   // mirror inside the row of 16 lanes: the other half's sum
        const float dDt = -dot / inv[i];
        if (cc == 0) {
          wl[buf][r] = cvt_bf16(dDt);
          dsum += dDt;
          if (blockIdx.y == 0 && (!RAGGED || t_stash + r < n)) dDout[(int64_t)slice * n + t_stash + r] = dDt;
        }
      }
    } else if (tid < 64) {
      wl[buf][tid] = cvt_bf16(wv);
    }
  };

  if (steps > 0) {
    fetch(t_begin);
    stash(0);
  }
  __syncthreads();
  // FUSE: rows 32 (wave / 2) + l32 of G are this wave's B operands in every step: kept in
  // registers (high part for the four k-steps, low part for the two of the quarter's own half).
  // The k-steps are taken own half first (ks_own, ks_own + 1: high and low part), then the other
  // half (high part only), so that the step loop has no branch and its LDS reads go out together.
  bf16x8 ghi[4], glo[2];
  const int ks_own = 2 * (wave >> 1), ks_oth = ks_own ^ 2;
  if (FUSE) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      ghi[u] = filter_operand(gt, 0, 32 * (wave >> 1) + l32, 2 * (ks_own + u) + h);
      ghi[2 + u] = filter_operand(gt, 0, 32 * (wave >> 1) + l32, 2 * (ks_oth + u) + h);
      glo[u] = filter_operand(gt, 1, 32 * (wave >> 1) + l32, 2 * (ks_own + u) + h);
    }
  }
  for (int s = 0; s < steps; ++s) {
    const int buf = s & 1;
    const bool more = s + 1 < steps;
    if (more) {
      t_stash = t_begin + 64 * (s + 1);
      fetch(t_stash);
    }
    if (FUSE) {
      // X_F^T quarter: columns 32 (wave % 2) .. + 31 of the tile, rows 32 (wave / 2) .. + 31.
      const bf16_t *raw = reinterpret_cast<const bf16_t *>(&xt[buf][0]);
      f32x16 q = zero16(), q2 = zero16();
      if (DEEP) {   // register i is column 32 (wave % 2) + acc_row(i, h) for every row of the quarter
        const float *ta = tile_add + ((int64_t)slice * ((n + 63) / 64) + (t_begin / 64 + s)) * DH + 32 * (wave & 1);
#pragma unroll
        for (int i = 0; i < 16; ++i) q[i] = ta[acc_row(i, h)];
      }
      bf16x8 xa[4];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        xa[u] = tile_cols_operand<false>(raw, XS, 32 * (wave & 1), ks_own + u, lane);
        xa[2 + u] = tile_cols_operand<false>(raw, XS, 32 * (wave & 1), ks_oth + u, lane);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {   // the low part matters inside the quarter's own 32-row half only
        q = mfma_bf16(xa[u], ghi[u], q);
        q2 = mfma_bf16(xa[u], glo[u], q2);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) q = mfma_bf16(xa[2 + u], ghi[2 + u], q);
#pragma unroll
      for (int i = 0; i < 16; ++i) q[i] += q2[i];
      // accumulator register i is column 32 (wave % 2) + acc_row(i, h), lane l32 is row 32 (wave / 2) + l32
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
        f16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (_Float16)q[4 * g + e];
        *reinterpret_cast<f16x4 *>(&xq[(32 * (wave >> 1) + l32) * XS + 32 * (wave & 1) + 8 * g + 4 * h]) = pk;
      }
      __syncthreads();
    }
    const _Float16 *xcur = FUSE ? &xq[0] : &xt[buf][0];
    __builtin_amdgcn_s_setprio(3);   // the matrix phase goes ahead of the other workgroup's tile traffic (-1 %)
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
      f16x8 xa[KS];   // projection A operand: rows 32 ti + l32, k = 8h + q (+16 per k-step)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        xa[ks] = *reinterpret_cast<const f16x8 *>(&xcur[(32 * ti + l32) * XS + 16 * ks + 8 * h]);
      bf16x8 yb[2][CT], wp[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        wp[a] = lds_perm8(&wl[buf][0], 32 * ti + 16 * a, h);
        // k-slot (h, q) of the chained MFMA stands for row 16 a + 8 (q / 4) + 4 h + (q % 4): two
        // transposing reads of four consecutive rows each, at column 32 ct + l32.
        const int i16 = lane & 15, c16 = 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
        const int trow = 32 * ti + 16 * a + 4 * h + (i16 >> 2);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          const bf16x4 lo = lds_read_tr4(&yt[buf][trow * YS + 32 * ct + c16]);
          const bf16x4 hi = lds_read_tr4(&yt[buf][(trow + 8) * YS + 32 * ct + c16]);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            yb[a][ct][q] = lo[q];
            yb[a][ct][4 + q] = hi[q];
          }
        }
      }
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        f32x16 R = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) R = mfma_f16(xa[ks], om[rt][ks], R);
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const bf16x8 pa = relu_bf16x8(pack_half(R, a));
          zacc[rt] = dot8_bf16(pa, wp[a], zacc[rt]);
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) S[rt][ct] = mfma_bf16(pa, yb[a][ct], S[rt][ct]);
        }
      }
    }
    __builtin_amdgcn_s_setprio(0);
    if (more) stash(buf ^ 1);
    __syncthreads();
  }
  float *sp = Spart + ((int64_t)slice * chunks + chunk) * (int64_t)m * DH;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        sp[(int64_t)(f0 + 32 * rt + acc_row(i, h)) * DH + 32 * ct + l32] = S[rt][ct][i];
    const float zt = xor32_sum(zacc[rt]);
    if (h == 0) zpart[((int64_t)slice * chunks + chunk) * m + f0 + 32 * rt + l32] = zt;
  }
  if (PREP && blockIdx.y == 0) {   // sum of dD over this chunk's rows, fixed order
    __shared__ float red[4];
    const float wsum = wave_sum64(dsum);
    if (lane == 0) red[wave] = wsum;
    __syncthreads();
    if (tid == 0) dDpart[(int64_t)slice * chunks + chunk] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

// M[slice][e] = scale[slice] * sum_chunk part[slice][chunk][e]  (e over m*DH; scale_ptr points at the
// slice rows' c * 2^-k entries, kCoefStride apart) and the vector part
// b likewise; plus the bf16 MFMA operand copies:
//   Mx  [m][DH+16]: row r = (M[r][0..DH), b[r], 0 x 15)   (A operand of dPhi = Y M^T + a b^T)
//   MT  [DH][m]   : M transposed                           (B operand of Phi M)
//   bb  [m]       : b in bf16
// One workgroup = 64 consecutive outputs x 4 waves; wave g sums the chunks g, g+4, ... with up
// to 16 loads in flight, the four partial sums meet in LDS in a fixed order.  Workgroups
// [0, m*DH/64) handle M, the next m/64 handle b.
template <int DH>
__global__ __launch_bounds__(256) void reduce_contract_kernel(const float *Spart, const float *zpart,
                                                             int chunks, int m, const float *scale_ptr,
                                                             float *S, float *z, bf16_t *Mx, bf16_t *MT,
                                                             bf16_t *bb) {
  constexpr int DX = DH + 16;
  const int slice = blockIdx.y, lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int64_t W = (int64_t)m * DH;
  const int wblocks = (int)(W / 64);
  const bool is_z = (int)blockIdx.x >= wblocks;
  const int64_t count = is_z ? m : W;
  const int64_t e = (is_z ? (int64_t)(blockIdx.x - wblocks) : (int64_t)blockIdx.x) * 64 + lane;
  const float *p = (is_z ? zpart : Spart) + (int64_t)slice * chunks * count + e;
  float acc = 0.f;
  int c = grp;
  for (; c + 60 < chunks; c += 64) {
    float v16[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v16[u] = p[(int64_t)(c + 4 * u) * count];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc += v16[u];
  }
  for (; c < chunks; c += 4) acc += p[(int64_t)c * count];
  __shared__ float part[4][64];
  part[grp][lane] = acc;
  __syncthreads();
  if (grp != 0) return;
  acc = ((part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane])) * scale_ptr[slice * kCoefStride];
  const bf16_t b = f32_to_bf16(acc);
  if (!is_z) {
    S[(int64_t)slice * W + e] = acc;
    const int r = (int)(e / DH), cidx = (int)(e % DH);
    Mx[((int64_t)slice * m + r) * DX + cidx] = b;
    MT[(int64_t)slice * W + (int64_t)cidx * m + r] = b;
  } else {
    z[(int64_t)slice * m + e] = acc;
    bb[(int64_t)slice * m + e] = b;
    bf16_t *ext = Mx + ((int64_t)slice * m + e) * DX + DH;
    ext[0] = b;
#pragma unroll
    for (int q = 1; q < 16; ++q) ext[q] = 0;
  }
}

// ------------------------------------------------------------------------------------
// rows kernel. One wave owns 64 consecutive rows at a time (one Haar block of the largest
// size); the workgroup's waves share the feature-side operands in LDS and walk over the
// row groups of their slice (the operands are staged once when all features fit).  The
// projection is computed transposed (features on the accumulator's register index, rows on
// lanes) so that the ReLU output chains into MFMAs that contract over the features.
//   MODE 0 (forward, Q side):   N = relu(R) S,  D = c * relu(R) z + eps,  O = c N / D
//   MODE 1 (backward, Q side):  G = dN S^T + dD z^T; dR = 1[R>0] G; dX_F = c dR Omega^T
//   MODE 2 (backward, K side):  G = V dS^T + 1 dz^T; dR, dX_F as above
//   MODE 3 (backward, K side):  dV = c relu(R) dS  (apply form, like MODE 0 without the normaliser)
// The rank-one term a b^T of G rides along as one extra k-step of the dPhi MFMA (operand
// rows extended by (b_r, 0, ...) and (a_t, 0, ...)).
// Backward epilogue: dX = gated Haar filter of dX_F (block-mean form on the accumulator
// layout, rows on registers), per-band inner products with X for dF, bf16 stores.
// ------------------------------------------------------------------------------------

// LN (MODE 0): LayerNorm over the columns of a row instead of the normaliser.  RAGGED: n is not a
// multiple of 64; rows past n of the last block read as zeros (clamped address, value replaced)
// and that block's output goes through a side buffer.  The plain instance has none of that code.
// DEEP: L > 6: X_F starts from the per-tile addend of the levels above 6 (tile_add
// [slices][ceil(n / 64)][DH]; head dimension 128 finds them in xf already); the gradient modes also
// write the 64-row sums of dX_F per column (tile_gsum, same shape) and leave band 6 of their
// partials as u_6 alone.
// DV (MODE 2, head dimension 64): the kernel also forms dV = c relu(R) dS of MODE 3 from the
// projection it has in hand (B operand: the rows of (dS | dz) in LDS through transposing reads)
// and writes it to out1; the separate MODE 3 launch, its pass over K and its projection go away.
template <int DH, int MODE, int NW, int MC, bool LN, bool RAGGED, bool DEEP, bool DV = false>
__global__ __launch_bounds__(NW * 64, NW == 8 ? 2 : 1) void rows_kernel(
    const _Float16 *xf,        // X_F fp16 [slices][n][DH] (head dimension 128; with 64 it is formed here)
    const bf16_t *x, View vx,  // X (Q or K): band inner products (MODE 1, 2); source of X_F (head dimension 64)
    const bf16_t *y, View vy,  // dO (MODE 1) or V (MODE 2)
    const float *Dsaved,       // D [slices][n] (MODE 1)
    const float *arow,         // dD [slices][n] (MODE 1)
    const _Float16 *omT,       // Omega^T fp16 [m][DH]
    const bf16_t *omega,       // Omega bf16 [DH][m]
    const bf16_t *Mx,          // (S | z) (MODE 1) / (dS | dz) (MODE 2), bf16 [slices][m][DH+16]
    const bf16_t *MT,          // S^T (MODE 0) / dS^T (MODE 3), bf16 [slices][DH][m]
    const bf16_t *bb,          // z bf16 [slices][m] (MODE 0)
    const float *coef,         // block-mean filter coefficients [slices][kCoefStride]
    const float *scalars, float eps, int n, int m, int row_groups,
    bf16_t *out0, View vo,     // O (MODE 0) / dQ or dK (MODE 1, 2) / dV (MODE 3)
    float *Dout,               // D (MODE 0)
    float *partF, int L,       // [slices][gridDim.x][L+1] band partials (MODE 1, 2)
    bf16_t *tail_out, float *tail_D,   // partial last block: its 64 output rows [slices][64][DH] and D [slices][64]
    const float *tile_add, float *tile_gsum,   // DEEP (see above)
    bf16_t *out1)                              // DV: dV, laid out like out0
{
  static_assert(!DV || (MODE == 2 && DH == 64 && NW == 4 && MC == 256), "dV rides along with the K-side gradient only");
  constexpr int KS = DH / 16, CT = DH / 32;
  constexpr int KSX = KS + 1;           // k-steps of the dPhi MFMA incl. the rank-one extension
  constexpr int AS = DH + 8;            // stride of the [feature][DH] fp16 array (16-byte reads)
  constexpr int AM = DH + 16 + 8;       // stride of the [feature][DH+16] bf16 array
  constexpr int NT = NW * 64;
  constexpr bool IS_GRAD = (MODE == 1 || MODE == 2);
  constexpr bool IS_APPLY = (MODE == 0 || MODE == 3);
  // Gradient modes run with the 512-register budget: projection and dPhi results go to VGPRs
  // where the register file has room for all their operands in VGPRs as well (head dimension 64
  // with the whole feature range staged; the other shapes keep the compiler's own allocation).
  constexpr bool VGPR_RG = IS_GRAD && NW == 4 && DH == 64 && MC == 256;
  // Head dimension 64: stage A runs here.  Each wave keeps the raw rows of its 64-row block in
  // LDS (one 64 x 32 panel per column tile), forms X_F^T = X^T G^T with 16 MFMAs at the top of
  // the block and packs the result into the projection's fp16 operands; the gradient modes
  // read X for the band inner products from the same panels, and every mode sends its output
  // tiles through a panel once its X values are used up.
  constexpr bool FUSE = (DH == 64);
  constexpr int NWR = NW;               // row groups of 64 rows per workgroup step (one per wave)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  constexpr int mc = MC;
  constexpr int BS = MC + 4;            // stride of [DH][feature] arrays (8-byte permuted reads)
  _Float16 *s_omT = reinterpret_cast<_Float16 *>(smem_raw);                 // [mc][AS]
  unsigned char *p = smem_raw + (size_t)mc * AS * 2;
  bf16_t *s_Mx = nullptr, *s_MT = nullptr, *s_om = nullptr, *s_bb = nullptr;
  if (IS_GRAD) { s_Mx = reinterpret_cast<bf16_t *>(p); p += (size_t)mc * AM * 2; }   // [mc][AM]
  if (IS_APPLY) { s_MT = reinterpret_cast<bf16_t *>(p); p += (size_t)DH * BS * 2; }   // [DH][BS]
  if (IS_GRAD) { s_om = reinterpret_cast<bf16_t *>(p); p += (size_t)DH * BS * 2; }   // [DH][BS]
  if (MODE == 0) { s_bb = reinterpret_cast<bf16_t *>(p); p += (size_t)mc * 2; }        // [mc]
  float *s_wave = reinterpret_cast<float *>(p); p += (size_t)NW * 64 * 4;              // [waves][64]
  constexpr int TS = 36;                // row stride (elements) of the per-wave 64 x 32 epilogue tile
  constexpr int TT = 68;                // column stride (elements) of the same tile held transposed [32][64]
  bf16_t *s_tile = reinterpret_cast<bf16_t *>(p);            // [waves][64][TS]; FUSE: [waves][CT][64][TS]
  constexpr int PANELS = FUSE ? CT : 1;
  p += (size_t)NW * PANELS * 64 * TS * 2;
  bf16_t *s_T = reinterpret_cast<bf16_t *>(p);               // FUSE: filter operand table [2][512]

  const int slice = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const float cscale = coef[slice * kCoefStride + kCoefCscale];   // c * 2^-k of this slice (X_F carries 2^k)
  const int nchunks = m / mc;

  // Feature-side operands of features [m0, m0 + MC) into LDS: every piece count is a compile-time
  // constant, loads go out in batches of eight before the first LDS write.
  auto stage = [&](int m0) {
    constexpr int CPRX = DH / 8;          // 16-byte pieces per Omega^T row
    constexpr int CPRM = (DH + 16) / 8;   // 16-byte pieces per extended M row
    constexpr int CPC = MC / 4;           // 8-byte pieces per column row (padded stride is 8-byte aligned)
    constexpr int B = 8;
    for (int e0 = 0; e0 < MC * CPRX; e0 += NT * B) {
      u16x8 tmp[B];
#pragma unroll
      for (int u = 0; u < B; ++u) {
        const int e = e0 + NT * u + tid;
        if (e < MC * CPRX)
          tmp[u] = *reinterpret_cast<const u16x8 *>(omT + (int64_t)(m0 + e / CPRX) * DH + (e % CPRX) * 8);
      }
#pragma unroll
      for (int u = 0; u < B; ++u) {
        const int e = e0 + NT * u + tid;
        if (e < MC * CPRX) *reinterpret_cast<u16x8 *>(&s_omT[(e / CPRX) * AS + (e % CPRX) * 8]) = tmp[u];
      }
    }
    if (IS_GRAD) {
      for (int e0 = 0; e0 < MC * CPRM; e0 += NT * B) {
        u16x8 tmp[B];
#pragma unroll
        for (int u = 0; u < B; ++u) {
          const int e = e0 + NT * u + tid;
          if (e < MC * CPRM)
            tmp[u] = *reinterpret_cast<const u16x8 *>(Mx + ((int64_t)slice * m + m0 + e / CPRM) * (DH + 16) +
                                                      (e % CPRM) * 8);
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
          const int e = e0 + NT * u + tid;
          if (e < MC * CPRM) *reinterpret_cast<u16x8 *>(&s_Mx[(e / CPRM) * AM + (e % CPRM) * 8]) = tmp[u];
        }
      }
    }
    for (int e0 = 0; e0 < DH * CPC; e0 += NT * B) {
      bf16x4 t1[B];
#pragma unroll
      for (int u = 0; u < B; ++u) {
        const int e = e0 + NT * u + tid;
        if (e < DH * CPC) {
          const int cidx = e / CPC, cc = e % CPC;
          t1[u] = IS_APPLY ? *reinterpret_cast<const bf16x4 *>(MT + ((int64_t)slice * DH + cidx) * m + m0 + cc * 4)
                           : *reinterpret_cast<const bf16x4 *>(omega + (int64_t)cidx * m + m0 + cc * 4);
        }
      }
#pragma unroll
      for (int u = 0; u < B; ++u) {
        const int e = e0 + NT * u + tid;
        if (e < DH * CPC) {
          const int cidx = e / CPC, cc = e % CPC;
          if (IS_APPLY) *reinterpret_cast<bf16x4 *>(&s_MT[cidx * BS + cc * 4]) = t1[u];
          else *reinterpret_cast<bf16x4 *>(&s_om[cidx * BS + cc * 4]) = t1[u];
        }
      }
    }
    if (MODE == 0)
      for (int e = tid; e < MC; e += NT) s_bb[e] = bb[(int64_t)slice * m + m0 + e];
  };

  float u[kTileBands];   // u_l = sum over blocks of bs_l(g) * bs_l(x), this lane's share
#pragma unroll
  for (int l = 0; l < kTileBands; ++l) u[l] = 0.f;
  float cf[kTileBands];
  if (IS_GRAD) {
#pragma unroll
    for (int l = 0; l < kTileBands; ++l) cf[l] = coef[slice * kCoefStride + l];
  }

  if (FUSE) build_filter_table(s_T, coef + slice * kCoefStride, tid, NT);
  if (nchunks == 1) stage(0);
  if (FUSE || nchunks == 1) __syncthreads();

  // ---- per-wave row-side operands; the next row group's are fetched right after the feature
  // loop of the current one (their registers are free by then), so that the latency of these
  // loads hides behind the epilogue.
  f16x8 xb[2][KS];      // X_F rows: B operand of the transposed projection
  u16x8 xp[8];          // FUSE: raw X rows of the next block, 16-byte row-major pieces (row lane / 8 + 8 j, columns 8 (lane % 8) ..)
  bf16x8 yb[2][KSX];    // dO or V rows (+ the a_t extension): B operand of the dPhi MFMA
  float dval[2] = {1.f, 1.f};   // D of rows 32 ti + l32 (MODE 1)
  float aval[2] = {1.f, 1.f};   // dD of the same rows (MODE 1)
  auto zero_if = [](bool bad, auto v) {
    if (bad) {
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = 0;
    }
    return v;
  };
  auto load_rows = [&](int t0) {
    const int last = RAGGED ? n - t0 - 1 : 63;   // last row of this block that exists
    if (FUSE) {
      if (!RAGGED) {
        // one running pointer (eight separately scaled row offsets would each be kept in registers)
        const bf16_t *xsrc = x + vx.slice_base(slice) + (int64_t)(t0 + (lane >> 3)) * vx.sn + (lane & 7) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          xp[j] = *reinterpret_cast<const u16x8 *>(xsrc);
          xsrc += 8 * vx.sn;
        }
      } else {
        const bf16_t *xsrc = x + vx.slice_base(slice) + (int64_t)t0 * vx.sn + (lane & 7) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int row = (lane >> 3) + 8 * j;
          xp[j] = zero_if(row > last, *reinterpret_cast<const u16x8 *>(xsrc + (int64_t)min(row, last) * vx.sn));
        }
      }
    } else {
      const _Float16 *xs = xf + ((int64_t)slice * n + t0) * DH;
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        const int row = 32 * ti + l32, rc = RAGGED ? min(row, last) : row;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const f16x8 v = *reinterpret_cast<const f16x8 *>(xs + (int64_t)rc * DH + 16 * ks + 8 * h);
          xb[ti][ks] = RAGGED ? zero_if(row > last, v) : v;
        }
      }
    }
    if (IS_GRAD) {
      // MODE 1 works with the raw dO rows: G' = D_t * G (the extension carries dD_t * D_t), and
      // row t of dX_F is scaled by c / D_t at the end; MODE 2 scales by c (extension 1, or 0 for
      // a row past n, which must not pick up the vector part).
      const bf16_t *ys = y + vy.slice_base(slice);
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        const int row = 32 * ti + l32;
        const bool bad = RAGGED && row > last;
        const int t = t0 + (RAGGED ? min(row, last) : row);
        if (MODE == 1) {   // only requested here: used at the top of the next round (finish_rows)
          dval[ti] = Dsaved[(int64_t)slice * n + t];
          aval[ti] = arow[(int64_t)slice * n + t];
          if (bad) { dval[ti] = 1.f; aval[ti] = 0.f; }
        } else if (RAGGED) {
          aval[ti] = bad ? 0.f : 1.f;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 v = *reinterpret_cast<const bf16x8 *>(ys + (int64_t)t * vy.sn + 16 * ks + 8 * h);
          yb[ti][ks] = RAGGED ? zero_if(bad, v) : v;
        }
      }
    }
  };
  // The rank-one extension (a_t, 0, ...) of the dPhi operand, built when the values have landed.
  auto finish_rows = [&]() {
    if (IS_GRAD) {
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        bf16x8 ext = splat_bf16x8(0.f);
        if (h == 0) ext[0] = (__bf16)(MODE == 1 ? aval[ti] * dval[ti] : (RAGGED ? aval[ti] : 1.0f));
        yb[ti][KSX - 1] = ext;
      }
    }
  };
  // FUSE: the raw rows go from the registers into the wave's panels as soon as the panels are
  // free (end of the epilogue), so that they do not occupy registers during the feature loop.
  bf16_t *panels = s_tile + wave * (PANELS * 64 * TS);
  auto put_rows = [&]() {
    if (FUSE) {
      __builtin_amdgcn_wave_barrier();
      // a 16-byte piece lies inside one panel (columns 8 (lane % 8) .. + 7); two 8-byte writes
      // because odd panel rows are only 8-byte aligned
      bf16_t *dstp = panels + ((lane & 7) >> 2) * (64 * TS) + (lane >> 3) * TS + ((lane & 3) << 3);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
        u16x4 lo4, hi4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          lo4[q] = xp[j][q];
          hi4[q] = xp[j][4 + q];
        }
        *reinterpret_cast<u16x4 *>(dstp + 8 * j * TS) = lo4;
        *reinterpret_cast<u16x4 *>(dstp + 8 * j * TS + 4) = hi4;
      }
      __builtin_amdgcn_wave_barrier();
    }
  };
  {
    const int t_first = (blockIdx.x * NWR + wave) * 64;
    if ((int)blockIdx.x < row_groups && t_first < n) {
      load_rows(t_first);
      put_rows();
    }
  }
  // (Two waves per SIMD: the wave priorities set around the feature loop below are what lets one
  // wave's epilogue run under the other's matrix work; an explicit start delay for the second wave
  // group, used before the priorities were there, no longer gains anything.)

  for (int rg = blockIdx.x; rg < row_groups; rg += gridDim.x) {
    const int t0 = (rg * NWR + wave) * 64;
    const bool active = t0 < n;
    // A partial last block (n not a multiple of 64) writes all its 64 rows to a side buffer, from
    // which a small kernel copies the rows that exist: the stores themselves stay unguarded
    // (guards or pointer selects around them cost the gradient kernels 230 bytes of spills per lane).
    const int valid = RAGGED ? n - t0 : 64;
    const bool tail = RAGGED && valid < 64;

    bf16x4 xpiece[8];   // X tile of the band inner products (MODE 1, 2, head dimension 128), 8-byte row-major pieces
    auto load_xpiece = [&](int ct, bf16x4 *dst) {
      if (!RAGGED) {
        const bf16_t *xsrc = x + vx.slice_base(slice) + (int64_t)(t0 + (lane >> 3)) * vx.sn + 32 * ct + (lane & 7) * 4;
#pragma unroll
        for (int j = 0; j < 8; ++j) {   // one running pointer instead of eight scaled row offsets
          dst[j] = *reinterpret_cast<const bf16x4 *>(xsrc);
          xsrc += 8 * vx.sn;
        }
      } else {
        const bf16_t *xsrc = x + vx.slice_base(slice) + (int64_t)t0 * vx.sn + 32 * ct + (lane & 7) * 4;
#pragma unroll
        for (int j = 0; j < 8; ++j) {   // rows past n: clamped address, value replaced by zeros
          const int row = (lane >> 3) + 8 * j;
          bf16x4 v4 = *reinterpret_cast<const bf16x4 *>(xsrc + (int64_t)min(row, valid - 1) * vx.sn);
          if (row >= valid) v4 = bf16x4{0, 0, 0, 0};
          dst[j] = v4;
        }
      }
    };
    if (FUSE && active) {
      // X_F^T = X^T G^T per (column tile, row tile) from the raw rows in the panels (written at
      // the end of the previous block's epilogue), then the projection's fp16 operands.
      __builtin_amdgcn_wave_barrier();
      // (apply modes: one column tile at a time, their 256-register budget has no room for four
      // accumulators next to the operands being built)
      constexpr int CG = IS_APPLY ? 1 : CT;   // column tiles per pass
#pragma unroll
      for (int c0 = 0; c0 < CT; c0 += CG) {
        f32x16 q[CG][2];
#pragma unroll
        for (int cg = 0; cg < CG; ++cg) {
          q[cg][0] = zero16();
          if (DEEP) {
            // register i stands for column 32 ct + (acc_row(i, h) with bits 2 and 3 swapped), every lane's row alike
            const float *ta = tile_add + ((int64_t)slice * ((n + 63) / 64) + t0 / 64) * DH + 32 * (c0 + cg);
#pragma unroll
            for (int i = 0; i < 16; ++i) q[cg][0][i] = ta[16 * (i >> 3) + 8 * h + 4 * ((i >> 2) & 1) + (i & 3)];
          }
          q[cg][1] = q[cg][0];
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          bf16x8 gop[2][2];
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            gop[tt][0] = filter_operand(s_T, 0, 32 * tt + l32, 2 * ks + h);
            gop[tt][1] = filter_operand(s_T, 1, 32 * tt + l32, 2 * ks + h);
          }
#pragma unroll
          for (int cg = 0; cg < CG; ++cg) {
            const bf16x8 xa = tile_cols_operand<true>(panels + (c0 + cg) * (64 * TS), TS, 0, ks, lane);
            // The low part matters inside the row tile's own 32-row half only: across the halves
            // every entry of G is the single coarsest-level coefficient.
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
              q[cg][tt] = mfma_bf16(xa, gop[tt][0], q[cg][tt]);
              if ((ks >> 1) == tt) q[cg][tt] = mfma_bf16(xa, gop[tt][1], q[cg][tt]);
            }
          }
        }
#pragma unroll
        for (int cg = 0; cg < CG; ++cg)
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            xb[tt][2 * (c0 + cg)] = pack_half_f16(q[cg][tt], 0);
            xb[tt][2 * (c0 + cg) + 1] = pack_half_f16(q[cg][tt], 1);
          }
      }
    }
    if (active) finish_rows();
    if (MODE == 1 && active) {   // row scales c / D_t for the epilogue, before the next rows' D replace them
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
        if (h == 0) s_wave[wave * 64 + 32 * ti + l32] = cscale * __builtin_amdgcn_rcpf(dval[ti]);
    }
    f32x16 acc0[2][CT];   // N, dV (MODE 0, 3) or dX_F (MODE 1, 2): rows on registers, columns on lanes
    f32x16 acc1[DV ? 2 : 1][DV ? CT : 1];   // DV: dV
    float dacc[2] = {0.f, 0.f};   // D partial of this lane's row (MODE 0)
#pragma unroll
    for (int ti = 0; ti < 2; ++ti)
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        acc0[ti][ct] = zero16();
        if (DV) acc1[ti][ct] = zero16();
      }

    for (int m0 = 0; m0 < m; m0 += mc) {
      if (nchunks > 1) {
        __syncthreads();
        stage(m0);
        __syncthreads();
      }
      if (!active) continue;

      if (VGPR_RG) {
        // The feature-side A operands of the next feature tile are read from LDS as soon as the
        // current tile's second chain has taken them.
        auto load_ops = [&](int rt, f16x8 *oa, bf16x8 *ma) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            oa[ks] = *reinterpret_cast<const f16x8 *>(&s_omT[(32 * rt + l32) * AS + 16 * ks + 8 * h]);
#pragma unroll
          for (int ks = 0; ks < KSX; ++ks)
            ma[ks] = *reinterpret_cast<const bf16x8 *>(&s_Mx[(32 * rt + l32) * AM + 16 * ks + 8 * h]);
        };
        // The B operands of what follows a chain are read from LDS BEFORE the chain's statement
        // (the compiler moves no LDS read across it): Omega[c][f] for dX_F, and for dV the rows of
        // (dS | dz) through transposing reads (k-slot (h, q) stands for feature
        // 32 rt + 16 a + 8 (q / 4) + 4 h + (q % 4): two reads of four consecutive rows each, at
        // column 32 ct + l32).  Both row tiles of a feature tile use the same operands.
        auto read_ob = [&](int rt, bf16x8 (*ob)[CT]) {
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
              ob[a][ct] = lds_perm8(&s_om[(32 * ct + l32) * BS], 32 * rt + 16 * a, h);
        };
        auto read_sb = [&](int rt, bf16x8 (*sb)[CT]) {
          const int i16 = lane & 15, c16 = 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
#pragma unroll
          for (int a = 0; a < 2; ++a) {
            const int frow = 32 * rt + 16 * a + 4 * h + (i16 >> 2);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
              const bf16x4 lo = lds_read_tr4(&s_Mx[frow * AM + 32 * ct + c16]);
              const bf16x4 hi = lds_read_tr4(&s_Mx[(frow + 8) * AM + 32 * ct + c16]);
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                sb[a][ct][q] = lo[q];
                sb[a][ct][4 + q] = hi[q];
              }
            }
          }
        };
        // What follows a masked chain: pack to bf16, dX_F += dR Omega^T (and dV += relu(R) dS).
        auto consume = [&](int ti, const f32x16 &Rt, const f32x16 &Gt, const bf16x8 (*ob)[CT],
                           const bf16x8 (*sb)[CT]) {
#pragma unroll
          for (int a = 0; a < 2; ++a) {
            const bf16x8 pg = pack_half(Gt, a);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc0[ti][ct] = mfma_bf16(pg, ob[a][ct], acc0[ti][ct]);
            if (DV) {
              const bf16x8 pa = relu_bf16x8(pack_half(Rt, a));
#pragma unroll
              for (int ct = 0; ct < CT; ++ct) acc1[ti][ct] = mfma_bf16(pa, sb[a][ct], acc1[ti][ct]);
            }
          }
        };
        // The pipelined form keeps two more chain results alive than the plain one: it is used where
        // the registers allow it without spills (not next to the dV accumulators, not with the
        // partial-block code).
        constexpr bool PIPE = !DV && !RAGGED;
        if (PIPE) {
          // Software pipeline over the feature tiles: while the matrix pipe works through the
          // chain of one row tile, the VALU masks the other row tile's finished chain (inside the
          // chain statements above); pack and dX_F MFMAs of a masked tile follow.  Per feature tile:
          //   chain of row tile 1 | mask of row tile 0, consume row tile 0,
          //   chain of row tile 0 of the NEXT feature tile | mask of row tile 1, consume row tile 1.
          constexpr int TILES = MC / 32;
          constexpr float kBig = 0x1p+100f;   // clamp(R * 2^100, 0, 1) = 1[R > 0] for every R > 2^-100
          f16x8 oa[KS];     // Omega^T rows of a feature tile: A operand of the projection
          bf16x8 ma[KSX];   // (M | b) rows of the same tile: A operand of the dPhi MFMA
          bf16x8 ob[2][CT];
          f32x16 R0, G0, R1, G1;
          load_ops(0, oa, ma);
          chain0_first(R0, G0, oa, xb[0], ma, yb[0]);
          for (int rt = 0; rt < TILES - 1; ++rt) {
            read_ob(rt, ob);
            chain1_mask0(R1, G1, G0, R0, oa, xb[1], ma, yb[1], kBig);
            load_ops(rt + 1, oa, ma);   // (lands while row tile 0 is consumed)
            consume(0, R0, G0, ob, nullptr);
            chain0_mask1(R0, G0, G1, R1, oa, xb[0], ma, yb[0], kBig);
            consume(1, R1, G1, ob, nullptr);
          }
          {   // the last feature tile: no chain follows it
            read_ob(TILES - 1, ob);
            chain1_mask0(R1, G1, G0, R0, oa, xb[1], ma, yb[1], kBig);
            consume(0, R0, G0, ob, nullptr);
#pragma unroll
            for (int i = 0; i < 16; ++i) G1[i] *= __builtin_amdgcn_fmed3f(R1[i] * kBig, 0.f, 1.f);
            consume(1, R1, G1, ob, nullptr);
          }
        } else {
          // Both row tiles' chains first, then mask, pack and the MFMAs that follow, tile by tile.
          constexpr int TILES = MC / 32;
          f16x8 oa[KS];
          bf16x8 ma[KSX];
          load_ops(0, oa, ma);
          for (int rt = 0; rt < TILES; ++rt) {
            bf16x8 ob[2][CT], sb[DV ? 2 : 1][CT];
            read_ob(rt, ob);
            if (DV) read_sb(rt, sb);
            f32x16 Rv[2], Gv[2];
            chain_first(Rv[0], Gv[0], oa, xb[0], ma, yb[0]);
            chain_first(Rv[1], Gv[1], oa, xb[1], ma, yb[1]);
            load_ops((rt + 1) & (TILES - 1), oa, ma);   // (the last round re-reads tile 0: in bounds, unused)
#pragma unroll
            for (int ti = 0; ti < 2; ++ti) {
#pragma unroll
              for (int i = 0; i < 16; ++i)
                Gv[ti][i] *= __builtin_amdgcn_fmed3f(Rv[ti][i] * 0x1p+100f, 0.f, 1.f);
              consume(ti, Rv[ti], Gv[ti], ob, sb);
            }
          }
        }
        continue;
      }
      // Head dimension 128, gradient modes: a bound the compiler cannot see keeps the loop rolled
      // (unrolled, the operands of several feature tiles are fetched ahead and spill).
      int rt_end = mc / 32;
      if (IS_GRAD && DH == 128) asm volatile("" : "+s"(rt_end));
      // Two waves per SIMD: the wave in its feature loop goes first, so that the other wave's epilogue
      // (no matrix work) fills the gaps instead of competing for issue slots (forward kernel -3 %).
      if (NW == 8) __builtin_amdgcn_s_setprio(3);
      for (int rt = 0; rt < rt_end; ++rt) {
        f16x8 oa[KS];     // Omega^T rows of this feature tile: A operand of the projection
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          oa[ks] = *reinterpret_cast<const f16x8 *>(&s_omT[(32 * rt + l32) * AS + 16 * ks + 8 * h]);
        bf16x8 ma[KSX];   // (M | b) rows of this feature tile: A operand of the dPhi MFMA
        if (IS_GRAD) {
#pragma unroll
          for (int ks = 0; ks < KSX; ++ks)
            ma[ks] = *reinterpret_cast<const bf16x8 *>(&s_Mx[(32 * rt + l32) * AM + 16 * ks + 8 * h]);
        }
#pragma unroll
        for (int ti = 0; ti < 2; ++ti) {
          f32x16 R = zero16();
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) R = mfma_f16(oa[ks], xb[ti][ks], R);
          if (IS_APPLY) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
              const bf16x8 pa = relu_bf16x8(pack_half(R, a));
              if (MODE == 0) dacc[ti] = dot8_bf16(pa, lds_perm8(s_bb, 32 * rt + 16 * a, h), dacc[ti]);
#pragma unroll
              for (int ct = 0; ct < CT; ++ct) {
                const bf16x8 sb = lds_perm8(&s_MT[(32 * ct + l32) * BS], 32 * rt + 16 * a, h);
                acc0[ti][ct] = mfma_bf16(pa, sb, acc0[ti][ct]);
              }
            }
          } else {
            f32x16 G = zero16();
#pragma unroll
            for (int ks = 0; ks < KSX; ++ks) G = mfma_bf16(ma[ks], yb[ti][ks], G);
            // 1[R > 0] as a multiplier without going through the condition register:
            // clamp(R * 2^100, 0, 1) is 1 for every R > 2^-100 and 0 for R <= 0.
#pragma unroll
            for (int i = 0; i < 16; ++i)
              G[i] *= __builtin_amdgcn_fmed3f(R[i] * 0x1p+100f, 0.f, 1.f);
#pragma unroll
            for (int a = 0; a < 2; ++a) {
              const bf16x8 pg = pack_half(G, a);
#pragma unroll
              for (int ct = 0; ct < CT; ++ct) {
                const bf16x8 ob = lds_perm8(&s_om[(32 * ct + l32) * BS], 32 * rt + 16 * a, h);
                acc0[ti][ct] = mfma_bf16(pg, ob, acc0[ti][ct]);
              }
            }
          }
        }
      }
    }
    if (NW == 8) __builtin_amdgcn_s_setprio(0);
    if (!active) continue;

    // ---- epilogues -----------------------------------------------------------------
    {
      // Unconditional (the last round re-requests its own rows): a branch around these loads
      // would leave two paths with different numbers of outstanding memory operations, and the
      // waits the compiler then places further down would cover the loads just issued.
      const int t_next = ((rg + gridDim.x) * NWR + wave) * 64;
      load_rows((rg + (int)gridDim.x < row_groups && t_next < n) ? t_next : t0);
    }
    bf16_t *tl = panels;   // FUSE, gradient modes: moves to the panel of the column tile in hand
    // Gradient modes: output tiles leave through the wave's LDS tile held transposed ([column][row]): a lane
    // stores its four consecutive accumulator rows as one 8-byte write, and transposing reads
    // hand back 8-byte row-major pieces (read u: rows 16 (u % 4) + lane % 16, columns
    // 16 (u / 4) + 4 (lane / 16) .. + 3) for the global stores.
    const int i16 = lane & 15, g16 = lane >> 4;
    auto tile_put = [&](int ti, const float *v16) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (__bf16)v16[4 * g + e];
        *reinterpret_cast<bf16x4 *>(&tl[l32 * TT + 32 * ti + 8 * g + 4 * h]) = pk;
      }
    };
    auto tile_store = [&](bf16_t *dst, int64_t sn, int col0) {
      bf16x4 piece[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        piece[u] = lds_read_tr4(&tl[(16 * (u >> 2) + 4 * g16 + (i16 >> 2)) * TT + 16 * (u & 3) + 4 * (i16 & 3)]);
      bf16_t *drow = dst + (int64_t)i16 * sn + col0 + 4 * g16;
#pragma unroll
      for (int u = 0; u < 4; ++u) {   // one running pointer instead of four scaled row offsets
        *reinterpret_cast<bf16x4 *>(drow) = piece[u];
        *reinterpret_cast<bf16x4 *>(drow + 16) = piece[u + 4];
        drow += 16 * sn;
      }
    };
    const int prow = lane >> 3, pcol = (lane & 7) * 4;   // this lane's 8-byte piece: rows prow + 8 j
    bf16_t *os = tail ? tail_out + (int64_t)slice * 64 * DH : out0 + vo.slice_base(slice) + (int64_t)t0 * vo.sn;
    const int64_t osn = tail ? DH : vo.sn;   // row stride of the output rows
    float *Dp = tail ? tail_D + slice * 64 : Dout + (int64_t)slice * n + t0;
    // DV: the second output's rows (side buffer: behind the first output's, [2][slices][64][DH])
    bf16_t *os1 = !DV ? nullptr
                      : (tail ? tail_out + ((int64_t)gridDim.y + slice) * 64 * DH
                              : out1 + vo.slice_base(slice) + (int64_t)t0 * vo.sn);

    if (MODE == 0 && LN) {
      // Output stage of Algorithm 1: O_t = (N_t - mean N_t) / sqrt(var N_t + eps), N = c * acc.
      // A row lives on one register index across the 32 lanes of a half-wave (and the CT column
      // tiles): mean first, then the centred second moment.  1 / sqrt(var + eps) goes to D.
      float *dl = s_wave + wave * 64;
#pragma unroll
      for (int ti = 0; ti < 2; ++ti)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float v = 0.f;
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) v += acc0[ti][ct][i];
          const float mu = half_wave_sum(v) * (1.0f / (float)DH);
          float q = 0.f;
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) {
            const float e = (acc0[ti][ct][i] - mu) * cscale;
            acc0[ti][ct][i] = e;
            q = fmaf(e, e, q);
          }
          const float rstd = 1.0f / sqrtf(half_wave_sum(q) * (1.0f / (float)DH) + eps);
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) acc0[ti][ct][i] *= rstd;
          if (l32 == 0) dl[32 * ti + acc_row(i, h)] = rstd;
        }
      __builtin_amdgcn_wave_barrier();
      Dp[lane] = dl[lane];
    } else if (MODE == 0) {   // normaliser D_t = c * sum_r relu(R) z + eps, row scale c / D_t
      float *dl = s_wave + wave * 64;
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        const float dsum = xor32_sum(dacc[ti]);
        const float Dt = fmaf(cscale, dsum, eps);
        // both half-waves hold the same sum and write the same values: no branch around the store
        dl[32 * ti + l32] = cscale * __builtin_amdgcn_rcpf(Dt);
        Dp[32 * ti + l32] = Dt;
      }
    }
    // Row scale of the accumulators (rows on registers): c / D_t (MODE 0 from the per-wave LDS
    // array written just above; LDS operations of one wave stay in order; MODE 1 from D), or c.
    __builtin_amdgcn_wave_barrier();
    if (!(MODE == 0 && LN))
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
      float sc[16];
      if (MODE == 0 || MODE == 1) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 s4 = *reinterpret_cast<const f32x4 *>(&s_wave[wave * 64 + 32 * ti + 8 * g + 4 * h]);
#pragma unroll
          for (int q = 0; q < 4; ++q) sc[4 * g + q] = s4[q];
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[i] = cscale;
      }
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc0[ti][ct][i] *= sc[i];
    }

    if (IS_APPLY) {   // O (MODE 0) or dV (MODE 3): bf16 through the wave's LDS tile, 8-byte row-major stores
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ti = 0; ti < 2; ++ti)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            tl[(32 * ti + acc_row(i, h)) * TS + l32] = cvt_bf16(acc0[ti][ct][i]);
        __builtin_amdgcn_wave_barrier();
        bf16x4 piece[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
          piece[j] = *reinterpret_cast<const bf16x4 *>(&tl[(prow + 8 * j) * TS + pcol]);
        bf16_t *orow = os + (int64_t)prow * osn + 32 * ct + pcol;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          *reinterpret_cast<bf16x4 *>(orow) = piece[j];
          orow += 8 * osn;
        }
      }
      put_rows();
      continue;
    }

    // MODE 1, 2: gated Haar filter of dX_F on the accumulator layout and band inner products.
    // Lane (l32, h) holds column 32 ct + l32 and rows 32 ti + 8 g + 4 h + e (g, e = 0..3):
    //   block sums of 2 and 4 rows are in-lane, 8 rows need the other half-wave (lane ^ 32),
    //   16 and 32 rows are in-lane again over g, 64 rows over ti.
    // X comes in and dX goes out through a wave-private LDS tile of 64 rows x 32 columns, so
    // that global memory sees 8-byte row-major accesses and the column accesses stay in LDS.
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      // ---- X tile -> LDS (FUSE: it is there already, in this column tile's panel)
      if (FUSE) {
        tl = panels + ct * (64 * TS);
      } else {
        load_xpiece(ct, xpiece);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < 8; ++j)
          *reinterpret_cast<bf16x4 *>(&tl[(prow + 8 * j) * TS + pcol]) = xpiece[j];
        __builtin_amdgcn_wave_barrier();
      }
      // ---- pass 1: block sums of g and x, band inner products, keep the 32-row sums
      float g5[2], x5[2];
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        float g1[8], x1[8];
        bf16x4 xq[4];   // X at this lane's accumulator positions: rows 8 g + 4 h + e of column l32
#pragma unroll
        for (int g = 0; g < 4; ++g)
          xq[g] = lds_read_tr4(&tl[(32 * ti + 8 * g + 4 * h + (i16 >> 2)) * TS + 16 * (g16 & 1) + 4 * (i16 & 3)]);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float ga = acc0[ti][ct][2 * k], gb = acc0[ti][ct][2 * k + 1];
          const float xa = (float)xq[k >> 1][2 * (k & 1)];
          const float xb2 = (float)xq[k >> 1][2 * (k & 1) + 1];
          u[0] = fmaf(ga, xa, fmaf(gb, xb2, u[0]));
          g1[k] = ga + gb;
          x1[k] = xa + xb2;
          u[1] = fmaf(g1[k], x1[k], u[1]);
        }
        float g3[4], x3[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float g2 = g1[2 * k] + g1[2 * k + 1], x2 = x1[2 * k] + x1[2 * k + 1];
          u[2] = fmaf(g2, x2, u[2]);
          g3[k] = xor32_sum(g2);   // 8-row blocks: both half-waves hold the same sums
          x3[k] = xor32_sum(x2);
          u[3] = fmaf(0.5f * g3[k], x3[k], u[3]);
        }
        const float g4a = g3[0] + g3[1], g4b = g3[2] + g3[3];
        const float x4a = x3[0] + x3[1], x4b = x3[2] + x3[3];
        u[4] = fmaf(0.5f * g4a, x4a, fmaf(0.5f * g4b, x4b, u[4]));
        g5[ti] = g4a + g4b;
        x5[ti] = x4a + x4b;
        u[5] = fmaf(0.5f * g5[ti], x5[ti], u[5]);
      }
      const float g6 = g5[0] + g5[1], x6 = x5[0] + x5[1];
      u[6] = fmaf(0.5f * g6, x6, u[6]);
      // both half-waves hold the same sum and write the same value: no branch around the store
      if (DEEP) tile_gsum[((int64_t)slice * ((n + 63) / 64) + t0 / 64) * DH + 32 * ct + l32] = g6;
      const float T6 = cf[6] * g6;
      __builtin_amdgcn_wave_barrier();
      // ---- pass 2: filtered gradient, top-down (block sums of g rebuilt), bf16 into the tile
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        const float T5 = fmaf(cf[5], g5[ti], T6);
        float g1[8], g2[4], g3[4], o16[16];
#pragma unroll
        for (int k = 0; k < 8; ++k) g1[k] = acc0[ti][ct][2 * k] + acc0[ti][ct][2 * k + 1];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          g2[k] = g1[2 * k] + g1[2 * k + 1];
          g3[k] = xor32_sum(g2[k]);
        }
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          const float T4 = fmaf(cf[4], g3[2 * k2] + g3[2 * k2 + 1], T5);
#pragma unroll
          for (int k1 = 0; k1 < 2; ++k1) {
            const int k = 2 * k2 + k1;   // 8-row block (and this lane's 4-row part of it)
            const float T2 = fmaf(cf[2], g2[k], fmaf(cf[3], g3[k], T4));
#pragma unroll
            for (int k0 = 0; k0 < 2; ++k0) {
              const int kk = 2 * k + k0;   // row pair
              const float T1 = fmaf(cf[1], g1[kk], T2);
#pragma unroll
              for (int e = 0; e < 2; ++e) {
                const int i = 2 * kk + e;
                o16[i] = fmaf(cf[0], acc0[ti][ct][i], T1);
              }
            }
          }
        }
        tile_put(ti, o16);
      }
      __builtin_amdgcn_wave_barrier();
      // ---- LDS -> dX
      tile_store(os, osn, 32 * ct);
      if (DV) {   // dV tile through the same panel (its X values are used up)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ti = 0; ti < 2; ++ti) {
          float o16[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) o16[i] = cscale * acc1[ti][ct][i];
          tile_put(ti, o16);
        }
        __builtin_amdgcn_wave_barrier();
        tile_store(os1, osn, 32 * ct);
      }
    }
    put_rows();
  }
  if (IS_APPLY) return;

  // With u_l = <dX_F, P_l X> (P_l = mean over aligned 2^l blocks) the band gradients are
  // dF_L = u_L and dF_{l-1} = u_{l-1} - u_l (l = 1..L); one partial per workgroup.
  __syncthreads();   // operand arrays are no longer read; s_wave is free for the reduction
#pragma unroll
  for (int l = 0; l < kTileBands; ++l) {
    const float s = wave_sum64(u[l]) / (float)(1 << l);
    if (lane == 0) s_wave[wave * 8 + l] = s;
  }
  __syncthreads();
  if (tid <= L) {
    // DEEP: levels above 6 are not seen here; band 6 keeps u_6 alone (its -u_7, and the bands
    // above, come from the tile-sum kernel in one extra row of the partials), bands above get 0.
    float ul = 0.f, ul1 = 0.f;
    if (tid < kTileBands)
      for (int wv = 0; wv < NW; ++wv) {
        ul += s_wave[wv * 8 + tid];
        if (tid < L && tid + 1 < kTileBands) ul1 += s_wave[wv * 8 + tid + 1];
      }
    const int rows = DEEP ? gridDim.x + DH / 16 : gridDim.x;   // (extra rows: one per workgroup of the tile-sum kernel)
    partF[((int64_t)slice * rows + blockIdx.x) * (L + 1) + tid] = tid < L ? ul - ul1 : ul;
  }
}

// dX[t][:] += dqbar / n (the pooled-query path; dqbar may be nullptr) + tile_add[t / 64][:] (the
// part of the gated filter above level 6; may be nullptr), bf16 read-modify-write with 16-byte
// accesses, four independent pieces per thread.
template <int DH, bool TILE>   // TILE: tile_add is given (the plain instance has none of its code)
__global__ __launch_bounds__(256) void add_pooled_kernel(bf16_t *dq, View v, const float *dqbar, int n,
                                                        float inv_n, const float *tile_add) {
  constexpr int CPR = DH / 8;
  const int slice = blockIdx.y;
  const int64_t total = (int64_t)n * CPR;
  const int64_t e0 = (int64_t)blockIdx.x * 1024 + threadIdx.x;
  const int cc = threadIdx.x % CPR;   // 256 and 1024 are multiples of CPR: same columns for all four
  const int ntiles = (n + 63) / 64;
  float add[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) add[q] = (!TILE || dqbar) ? dqbar[(int64_t)slice * DH + cc * 8 + q] * inv_n : 0.f;
  bf16_t *base = dq + v.slice_base(slice) + cc * 8;
  u16x8 val[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t e = e0 + 256 * u;
    if (e < total) val[u] = *reinterpret_cast<u16x8 *>(base + (e / CPR) * v.sn);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t e = e0 + 256 * u;
    if (e < total) {
      const int64_t row = e / CPR;
      float tadd[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (TILE) {   // two 16-byte loads of the tile's addend (32-byte aligned: DH and 8 cc are multiples of 8)
        const f32x4 *ta = reinterpret_cast<const f32x4 *>(tile_add + ((int64_t)slice * ntiles + (row >> 6)) * DH + cc * 8);
        const f32x4 t0 = ta[0], t1 = ta[1];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          tadd[q] = t0[q];
          tadd[4 + q] = t1[q];
        }
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) val[u][q] = f32_to_bf16(bf16_to_f32(val[u][q]) + add[q] + tadd[q]);
      *reinterpret_cast<u16x8 *>(base + row * v.sn) = val[u];
    }
  }
}

// ------------------------------------------------------------------------------------
// Transforms deeper than one 64-row block (L > 6).  In block-mean form the
// levels above 6 add, to every row of a tile, coef_l times the sum of X over the 2^l-row block
// that holds the tile: a per-(tile, column) addend built from the tile sums.
// Pyramid of one signal: level j (1 .. J) holds the sums over 2^j consecutive tiles,
// [ceil(ntiles / 2^j)][d], levels packed one after the other in P (< ntiles + J rows).
// d / 16 workgroups of 1024 threads per signal, one per 16 columns; thread (column c = tid % 16 of
// its 16, group g = tid / 16 of kCoarseGroups); the loops over tiles carry no dependency and
// are unrolled so that several loads are in flight.
// ------------------------------------------------------------------------------------
constexpr int kCoarseGroups = 64, kCoarseCols = 16;   // (the gradient rows kernel leaves d / 16 extra rows in its band partials)
__device__ __forceinline__ void build_tile_pyramid(const float *T, int ntiles, int d, int J, float *P, int c, int g) {
  const float *prev = T;
  int nprev = ntiles;
  float *cur = P;
  for (int j = 1; j <= J; ++j) {
    const int nb = (nprev + 1) / 2;
#pragma unroll 4
    for (int b = g; b < nb; b += kCoarseGroups)
      cur[b * d + c] = prev[2 * b * d + c] + (2 * b + 1 < nprev ? prev[(2 * b + 1) * d + c] : 0.f);
    __threadfence_block();
    __syncthreads();
    prev = cur;
    nprev = nb;
    cur += nb * d;
  }
}
// addend[tile][c] = sum over j of coef[6 + j] * P_j[tile >> j][c]
__device__ __forceinline__ void tile_addend(const float *P, const float *coef, int ntiles, int d, int J, float *A, int c, int g) {
#pragma unroll 4
  for (int tile = g; tile < ntiles; tile += kCoarseGroups) {
    float acc = 0.f;
    const float *lvl = P;
    int nprev = ntiles;
    for (int j = 1; j <= J; ++j) {
      const int nb = (nprev + 1) / 2;
      acc = fmaf(coef[6 + j], lvl[(tile >> j) * d + c], acc);
      lvl += nb * d;
      nprev = nb;
    }
    A[tile * d + c] = acc;
  }
}
constexpr int64_t pyramid_floats(int ntiles, int d) { return ((int64_t)ntiles + 32) * d; }

// Forward: blockIdx.y = 0 for Q, 1 for K; blockIdx.z = group of 16 columns.  T*: tile sums
// [S][ntiles][d]; A*: addends, same shape; pyr: 2 * S pyramids of pyramid_floats(ntiles, d).
__global__ __launch_bounds__(1024) void coarse_addend_kernel(const float *Tq, const float *Tk, const float *coef,
                                                            int ntiles, int d, int L, float *pyr, float *Aq, float *Ak) {
  const int slice = blockIdx.x, side = blockIdx.y;
  const int c = kCoarseCols * blockIdx.z + (threadIdx.x & (kCoarseCols - 1)), g = threadIdx.x / kCoarseCols;
  const int64_t base = (int64_t)slice * ntiles * d;
  float *P = pyr + ((int64_t)slice * 2 + side) * pyramid_floats(ntiles, d);
  build_tile_pyramid((side ? Tk : Tq) + base, ntiles, d, L - 6, P, c, g);
  tile_addend(P, coef + slice * kCoefStride, ntiles, d, L - 6, (side ? Ak : Aq) + base, c, g);
}

// Backward, after both gradient kernels: Tg* = tile sums of dX_F (written by their epilogues),
// Tx* = tile sums of X.  Writes the addends of dX (the filter is symmetric) and, into the extra
// rows row .. row + d / 16 - 1 (one per workgroup) of the band partials part*[S][row + d / 16][L + 1], the
// contribution of the levels above 6: with u_l = 2^-l * sum over 2^l-row blocks and columns of
// blocksum(dX_F) * blocksum(X), band 6 gets -u_7, band l (7 .. L-1) gets u_l - u_{l+1}, band L
// gets u_L (the gradient kernels leave u_6 alone in band 6 and zeros above).
__global__ __launch_bounds__(1024) void coarse_bwd_kernel(const float *TgQ, const float *TgK, const float *TxQ,
                                                         const float *TxK, const float *coef, int ntiles, int d, int L,
                                                         float *pyr, float *AQ, float *AK, float *partQ,
                                                         float *partK, int row) {
  const int slice = blockIdx.x, side = blockIdx.y, J = L - 6;
  const int c = kCoarseCols * blockIdx.z + (threadIdx.x & (kCoarseCols - 1)), g = threadIdx.x / kCoarseCols;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t base = (int64_t)slice * ntiles * d;
  float *Pg = pyr + (((int64_t)slice * 2 + side) * 2) * pyramid_floats(ntiles, d);
  float *Px = Pg + pyramid_floats(ntiles, d);
  build_tile_pyramid((side ? TgK : TgQ) + base, ntiles, d, J, Pg, c, g);
  build_tile_pyramid((side ? TxK : TxQ) + base, ntiles, d, J, Px, c, g);
  tile_addend(Pg, coef + slice * kCoefStride, ntiles, d, J, (side ? AK : AQ) + base, c, g);
  __shared__ float red[16];
  __shared__ float u[kMaxBands + 1];
  const float *lg = Pg, *lx = Px;
  int nprev = ntiles;
  for (int j = 1; j <= J; ++j) {
    const int nb = (nprev + 1) / 2;
    float acc = 0.f;
#pragma unroll 4
    for (int b = g; b < nb; b += kCoarseGroups) acc = fmaf(lg[b * d + c], lx[b * d + c], acc);
    acc = wave_sum64(acc);
    if (lane == 0) red[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      float tot = 0.f;
      for (int i = 0; i < 16; ++i) tot += red[i];
      u[6 + j] = tot / (float)(1 << (6 + j));
    }
    __syncthreads();
    lg += nb * d;
    lx += nb * d;
    nprev = nb;
  }
  if ((int)threadIdx.x <= L) {
    const int i = threadIdx.x;
    float val = 0.f;
    if (i == 6) val = -u[7];
    else if (i > 6) val = i < L ? u[i] - u[i + 1] : u[i];
    float *part = side ? partK : partQ;
    part[((int64_t)slice * (row + gridDim.z) + row + blockIdx.z) * (L + 1) + i] = val;
  }
}

// Backward of the LayerNorm output stage (Algorithm 1), row by row:
//   dN_t = rstd_t (dO_t - mean dO_t - O_t mean(dO_t * O_t))   -> bf16 [slices][n][DH]
// The gradient kernels then run as without a normaliser: D = 1 and dD = 0 (written here).
// part[slice][chunk] = sum over the chunk's rows of -<dO_t, O_t> rstd_t^2, the per-row term of
// d sigma (N scales with 1 / sigma^2 and <dN_t, N_t> = <dO_t, O_t> eps rstd_t^2).
// DH / 8 lanes share a row, 16 bytes each.
template <int DH>
__global__ __launch_bounds__(256) void ln_prep_kernel(const bf16_t *dout, const bf16_t *out, View v,
                                                     const float *rstd, int n, int rows_per_chunk,
                                                     bf16_t *dN, float *ones, float *zeros, float *part) {
  constexpr int CPR = DH / 8, RPB = 256 / CPR;
  const int slice = blockIdx.y, chunk = blockIdx.x, tid = threadIdx.x;
  const int t_begin = chunk * rows_per_chunk, t_end = min(n, t_begin + rows_per_chunk);
  const int r = tid / CPR, cc = tid % CPR;
  const int64_t base = v.slice_base(slice);
  float acc = 0.f;
  for (int t = t_begin + r; t < t_end; t += RPB) {
    const int64_t off = base + (int64_t)t * v.sn + cc * 8;
    const u16x8 g8 = *reinterpret_cast<const u16x8 *>(dout + off);
    const u16x8 o8 = *reinterpret_cast<const u16x8 *>(out + off);
    float g[8], o[8], sg = 0.f, sgo = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      g[q] = bf16_to_f32(g8[q]);
      o[q] = bf16_to_f32(o8[q]);
      sg += g[q];
      sgo = fmaf(g[q], o[q], sgo);
    }
#pragma unroll
    for (int d = 1; d < CPR; d <<= 1) {
      sg += __shfl_xor(sg, d, 64);
      sgo += __shfl_xor(sgo, d, 64);
    }
    const int64_t row = (int64_t)slice * n + t;
    const float rs = rstd[row];
    const float m1 = sg * (1.0f / (float)DH), m2 = sgo * (1.0f / (float)DH);
    u16x8 d8;
#pragma unroll
    for (int q = 0; q < 8; ++q) d8[q] = cvt_bf16(rs * (g[q] - m1 - o[q] * m2));
    *reinterpret_cast<u16x8 *>(dN + row * DH + cc * 8) = d8;
    if (cc == 0) {
      ones[row] = 1.0f;
      zeros[row] = 0.0f;
      acc -= sgo * rs * rs;
    }
  }
  acc = wave_sum64(acc);
  __shared__ float red[4];
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) part[(int64_t)slice * gridDim.x + chunk] = (red[0] + red[1]) + (red[2] + red[3]);
}

// Partial last block of a sequence: rows [t0, n) of the side buffer [slices][64][DH] (and of
// D [slices][64] when given) go to their place in the output.
template <int DH>
__global__ __launch_bounds__(256) void tail_copy_kernel(const bf16_t *tail_out, const float *tail_D, int n,
                                                       int t0, bf16_t *out, View v, float *D) {
  constexpr int CPR = DH / 8;
  const int slice = blockIdx.x, valid = n - t0;
  for (int e = threadIdx.x; e < valid * CPR; e += 256) {
    const int r = e / CPR, cc = e % CPR;
    *reinterpret_cast<u16x8 *>(out + v.slice_base(slice) + (int64_t)(t0 + r) * v.sn + cc * 8) =
        *reinterpret_cast<const u16x8 *>(tail_out + ((int64_t)slice * 64 + r) * DH + cc * 8);
  }
  if (D && (int)threadIdx.x < valid) D[(int64_t)slice * n + t0 + threadIdx.x] = tail_D[slice * 64 + threadIdx.x];
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
constexpr int kWavesGrad = 4;
constexpr int waves_apply(int d) { return d == 64 ? 8 : 4; }   // head dimension 128: 512 registers per lane

struct FastPlan {
  int DH, FW, MB, mc, mcA;   // features staged in LDS per pass by the rows kernels (mcA: the dV kernel)
  int chunksQ, rowsQ;   // pooled-query partial sums
  int chunksC, rowsC;   // split of n in phiT_contract
  int rowGroupsA, rowsWgsA;   // apply-type rows kernel (4 waves): row groups / workgroups per slice
  int rowGroupsG, rowsWgsG;   // gradient-type rows kernel (8 waves)
};

FastPlan fast_plan(const wersa_desc &c) {
  FastPlan p{};
  p.DH = c.d;
  if (c.m % 256 == 0 && c.d == 64) { p.FW = 64; p.MB = 256; } else { p.FW = 32; p.MB = 128; }
  p.mc = (c.d == 64 && c.m % 256 == 0) ? 256 : 128;
  // the dV kernel stages no (M | b) array: 256 features fit for head dimension 128 too (the forward
  // kernel, which could do the same, measured 3 % slower with 256 than with 128)
  p.mcA = c.m % 256 == 0 ? 256 : 128;
  const int slices = c.B * c.H, blocks = (c.n + 63) / 64;
  int cq = (c.n + 1023) / 1024;
  p.chunksQ = cq < 1 ? 1 : (cq > 512 ? 512 : cq);
  p.rowsQ = (c.n + p.chunksQ - 1) / p.chunksQ;
  p.chunksQ = (c.n + p.rowsQ - 1) / p.rowsQ;
  if (c.L > kTileL) {   // the pooled-query partial sums double as the 64-row tile sums
    p.rowsQ = 64;
    p.chunksQ = blocks;
  }
  int want = 512 / (slices * (c.m / p.MB));   // two resident workgroups per compute unit, one round
  if (want < 1) want = 1;
  if (want > blocks) want = blocks;
  const int bpc = (blocks + want - 1) / want;
  p.rowsC = bpc * 64;
  p.chunksC = (blocks + bpc - 1) / bpc;
  p.rowGroupsA = (blocks + waves_apply(c.d) - 1) / waves_apply(c.d);
  // One resident workgroup per compute unit (the operand arrays fill most of the LDS): at most
  // 256 workgroups in total, so that no second, mostly empty round follows the first.
  int wgs = 256 / slices < 1 ? 1 : 256 / slices;
  p.rowsWgsA = wgs < p.rowGroupsA ? wgs : p.rowGroupsA;
  p.rowGroupsG = (blocks + kWavesGrad - 1) / kWavesGrad;
  p.rowsWgsG = wgs < p.rowGroupsG ? wgs : p.rowGroupsG;
  return p;
}

struct FastWs {
  float *qamax;   // largest |Q| per (slice, chunk) of the pooling pass
  float *scalars, *coef, *qpart, *Spart, *zpart, *dD, *dDpart, *dS, *dz, *partQ, *partK, *dF,
      *dlogit, *dqbar;
  bf16_t *tail_out;   // partial last block of the sequence: its 64 output rows [slices][64][d]
  float *tail_D;      // and its D values [slices][64]
  _Float16 *omT;
  bf16_t *Sx, *ST, *zb, *dSx, *dST, *dzb;
  bf16_t *dN;    // LayerNorm output stage: gradient with respect to the un-normalised rows
  float *ones;   // and the stand-in for D in the gradient kernels
  // L > 6: tile sums of Q and K and the addends of the levels above 6 (saved buffer); tile sums
  // of dQ_F and dK_F, the addends of dQ and dK, and the pyramids (workspace)
  float *tileQ, *tileK, *addQ, *addK, *gsumQ, *gsumK, *gaddQ, *gaddK, *pyr;
  int64_t total;
};

// Workspace pieces; the per-call constants and the forward's bf16 operand copies live in the
// saved buffer (the backward reads them back instead of rebuilding them).
FastWs fast_ws(const wersa_desc &c, const FastPlan &p, int bwd, float *base, float *saved) {
  FastWs w{};
  Bump b(base);
  const int64_t sl = (int64_t)c.B * c.H, md = (int64_t)c.m * c.d;
  const SavedLayout sv = saved_layout(c);
  if (saved) {
    w.scalars = saved + sv.scalars;
    w.coef = saved + sv.coef;
    w.omT = reinterpret_cast<_Float16 *>(saved + sv.omT);
    w.Sx = reinterpret_cast<bf16_t *>(saved + sv.Sx);
    w.ST = reinterpret_cast<bf16_t *>(saved + sv.ST);
    w.zb = reinterpret_cast<bf16_t *>(saved + sv.zb);
    if (sv.tileQ >= 0) {
      w.tileQ = saved + sv.tileQ;
      w.tileK = saved + sv.tileK;
      w.addQ = saved + sv.addQ;
      w.addK = saved + sv.addK;
    }
  }
  const bool deep = c.L > kTileL;
  const int ntiles = (c.n + 63) / 64;
  w.tail_out = reinterpret_cast<bf16_t *>(b.take(2 * sl * 64 * c.d / 2));   // (two outputs when dV rides along with dK)
  w.tail_D = b.take(sl * 64);
  w.qpart = b.take(sl * p.chunksQ * c.d);
  w.qamax = b.take(sl * p.chunksQ);
  w.Spart = b.take(sl * p.chunksC * md);
  w.zpart = b.take(sl * p.chunksC * c.m);
  const int64_t mx = (int64_t)c.m * (c.d + 16);
  if (bwd) {
    w.dD = b.take(sl * c.n);
    w.dDpart = b.take(sl * p.chunksC);
    w.dS = b.take(sl * md);
    w.dz = b.take(sl * c.m);
    w.dSx = reinterpret_cast<bf16_t *>(b.take(sl * mx / 2));
    w.dST = reinterpret_cast<bf16_t *>(b.take(sl * md / 2));
    w.dzb = reinterpret_cast<bf16_t *>(b.take(sl * c.m / 2));
    w.partQ = b.take(sl * (p.rowsWgsG + c.d / kCoarseCols) * (c.L + 1));   // (+ the rows of the levels above 6)
    w.partK = b.take(sl * (p.rowsWgsG + c.d / kCoarseCols) * (c.L + 1));
    if (deep) {
      const int64_t tiles = sl * ntiles * c.d;
      w.gsumQ = b.take(tiles);
      w.gsumK = b.take(tiles);
      w.gaddQ = b.take(tiles);
      w.gaddK = b.take(tiles);
    }
    w.dF = b.take(sl * (c.L + 1));
    w.dlogit = b.take(sl * (c.L + 1));
    w.dqbar = b.take(sl * c.d);
    if (c.flags & WERSA_FLAG_LAYERNORM) {
      w.dN = reinterpret_cast<bf16_t *>(b.take(sl * c.n * c.d / 2));
      w.ones = b.take(sl * c.n);
    }
  }
  if (deep) w.pyr = b.take(sl * 4 * pyramid_floats(ntiles, c.d));
  w.total = b.off;
  return w;
}

template <int DH, int MODE, int NW>
size_t rows_smem_bytes(int mc) {
  constexpr bool IS_GRAD = (MODE == 1 || MODE == 2);
  const size_t AS = DH + 8, AM = DH + 16 + 8, BS = (size_t)mc + 4;
  size_t s = (size_t)mc * AS * 2;
  if (IS_GRAD) s += (size_t)mc * AM * 2 + (size_t)DH * BS * 2;
  else s += (size_t)DH * BS * 2;
  if (MODE == 0) s += (size_t)mc * 2;
  s += NW * 64 * 4;
  if (DH == 64) s += (size_t)NW * (DH / 32) * 64 * 36 * 2 + 2 * 512 * 2;   // X panels per wave and the filter table
  else s += (size_t)NW * 64 * 36 * 2;
  return s;
}

// dV formed by the K-side gradient kernel instead of a launch of its own: head dimension 64 with
// 256 features staged per pass, whole 64-row blocks (with a partial last block the merged kernel
// would spill ~100 bytes per lane; those shapes keep the two launches).
inline bool dv_rides_along(const wersa_desc &c, const FastPlan &p) {
  return c.d == 64 && p.mc == 256 && c.n % 64 == 0;
}

template <int DH, int MODE>
hipError_t launch_rows(const wersa_desc &c, const FastPlan &p, const _Float16 *xf, const bf16_t *x,
                       const bf16_t *y, const float *Dsaved, const float *arow, const FastWs &w,
                       const bf16_t *omega, const bf16_t *Mx, const bf16_t *MT, const bf16_t *bb,
                       bf16_t *out0, float *Dout, float *partF, hipStream_t st,
                       const View *yview = nullptr, bf16_t *out1 = nullptr) {
  constexpr bool IS_GRAD = (MODE == 1 || MODE == 2);
  constexpr int NW = IS_GRAD ? kWavesGrad : waves_apply(DH);
  // key-side modes take the second random matrix when the descriptor has two
  const int64_t side = ((c.flags & WERSA_FLAG_SEPARATE_OMEGA) && MODE >= 2) ? (int64_t)c.d * c.m : 0;
  const _Float16 *omT = w.omT + side;
  omega += side;
  const View tv{c.stride_b, c.stride_h, c.stride_n, c.H};
  const int mcs = MODE == 3 ? p.mcA : p.mc;
  // (the gradient kernels of head dimension 128 exist with 128 staged features only)
  constexpr int MCH = (DH == 128 && IS_GRAD) ? 128 : 256;
  const size_t smem = rows_smem_bytes<DH, MODE, NW>(mcs);
  const char *name = MODE == 0 ? "wersa_rows_fwd"
                               : (MODE == 1 ? "wersa_rows_bwd_q" : (MODE == 2 ? "wersa_rows_bwd_k" : "wersa_rows_bwd_v"));
  const int wgs = IS_GRAD ? p.rowsWgsG : p.rowsWgsA, groups = IS_GRAD ? p.rowGroupsG : p.rowGroupsA;
  auto go = [&](auto kern) -> hipError_t {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    WERSA_STAGE(name, st,
                kern<<<dim3(wgs, c.B * c.H), NW * 64, smem, st>>>(
                    xf, x, tv, y, yview ? *yview : tv, Dsaved, arow, omT, omega, Mx, MT, bb, w.coef, w.scalars,
                    c.eps, c.n, c.m, groups, out0, tv, Dout, partF, c.L, w.tail_out, w.tail_D,
                    MODE >= 2 ? w.addK : w.addQ, MODE == 1 ? w.gsumQ : w.gsumK, out1));
    if (c.n % 64 != 0) {
      WERSA_STAGE("wersa_tail_copy", st,
                  tail_copy_kernel<DH><<<c.B * c.H, 256, 0, st>>>(w.tail_out, MODE == 0 ? w.tail_D : nullptr, c.n,
                                                                   c.n / 64 * 64, out0, tv, Dout));
      if (out1)
        WERSA_STAGE("wersa_tail_copy", st,
                    tail_copy_kernel<DH><<<c.B * c.H, 256, 0, st>>>(w.tail_out + (int64_t)c.B * c.H * 64 * DH, nullptr, c.n,
                                                                     c.n / 64 * 64, out1, tv, nullptr));
    }
    return hipSuccess;
  };
  if (out1) {   // dV rides along with the K-side gradient (see dv_rides_along)
    constexpr bool OK = MODE == 2 && DH == 64;
    constexpr int MCV = OK ? 256 : 128;
    if (c.L > kTileL) return go(&rows_kernel<DH, MODE, NW, MCV, false, false, OK, OK>);
    return go(&rows_kernel<DH, MODE, NW, MCV, false, false, false, OK>);
  }
  const bool ln = MODE == 0 && (c.flags & WERSA_FLAG_LAYERNORM), ragged = c.n % 64 != 0;
  if (DH == 128 && IS_GRAD && c.L > kTileL) {
    // deeper than one block, head dimension 128: X_F arrives with the levels above 6 in it; the
    // gradient modes still write the tile sums of dX_F and the extra rows of the band partials
    if (ragged) return go(&rows_kernel<DH, MODE, NW, 128, false, DH == 128 && IS_GRAD, DH == 128 && IS_GRAD>);
    return go(&rows_kernel<DH, MODE, NW, 128, false, false, DH == 128 && IS_GRAD>);
  }
  if (DH == 64 && c.L > kTileL) {   // deeper than one block, head dimension 64
    if (ragged) {
      if (ln) return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, MODE == 0, DH == 64, DH == 64>)
                                 : go(&rows_kernel<DH, MODE, NW, 128, MODE == 0, DH == 64, DH == 64>);
      return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, false, DH == 64, DH == 64>)
                         : go(&rows_kernel<DH, MODE, NW, 128, false, DH == 64, DH == 64>);
    }
    if (ln) return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, MODE == 0, false, DH == 64>)
                               : go(&rows_kernel<DH, MODE, NW, 128, MODE == 0, false, DH == 64>);
    return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, false, false, DH == 64>)
                       : go(&rows_kernel<DH, MODE, NW, 128, false, false, DH == 64>);
  }
  if (ragged) {   // the shapes with a partial last block take the guarded instances
    if (ln) return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, MODE == 0, true, false>)
                               : go(&rows_kernel<DH, MODE, NW, 128, MODE == 0, true, false>);
    return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, false, true, false>)
                       : go(&rows_kernel<DH, MODE, NW, 128, false, true, false>);
  }
  if (ln) return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, MODE == 0, false, false>)
                             : go(&rows_kernel<DH, MODE, NW, 128, MODE == 0, false, false>);
  return mcs == 256 ? go(&rows_kernel<DH, MODE, NW, MCH, false, false, false>)
                     : go(&rows_kernel<DH, MODE, NW, 128, false, false, false>);
}

// orows != nullptr selects the backward form that derives dD from the rows of O itself;
// otherwise the row weights of the vector part are `wts` (all ones when nullptr).
template <int DH>
void launch_contract(const wersa_desc &c, const FastPlan &p, const _Float16 *xf, const bf16_t *xraw,
                     const bf16_t *y, const View &yv, const float *rowdiv, const float *wts, const bf16_t *orows,
                     bool key_side, const FastWs &w, float *S, float *z, bf16_t *Mx, bf16_t *MT,
                     bf16_t *bb, hipStream_t st) {
  const int slices = c.B * c.H;
  dim3 grid(p.chunksC, c.m / p.MB, slices);
  const _Float16 *omT = w.omT + (((c.flags & WERSA_FLAG_SEPARATE_OMEGA) && key_side) ? (int64_t)c.d * c.m : 0);
  auto go = [&](auto kern) {
    WERSA_STAGE("wersa_phiT_contract", st,
                kern<<<grid, 256, 0, st>>>(xf, xraw, View{c.stride_b, c.stride_h, c.stride_n, c.H}, w.coef,
                                           key_side ? w.addK : w.addQ, y, yv,
                                           rowdiv, wts, orows, w.dD, w.dDpart, omT, c.n, c.m, p.rowsC, w.Spart,
                                           w.zpart));
  };
  const bool ragged = c.n % 64 != 0, deep = DH == 64 && c.L > kTileL;
  constexpr int FWB = DH == 64 ? 64 : 32;   // 64 features per wave exist for head dimension 64 only (see fast_plan)
  constexpr bool D64 = DH == 64;
  const bool wide = p.FW == 64;
  if (deep && ragged) {
    if (wide) orows ? go(&phiT_contract_kernel<DH, FWB, true, D64, D64>) : go(&phiT_contract_kernel<DH, FWB, false, D64, D64>);
    else orows ? go(&phiT_contract_kernel<DH, 32, true, D64, D64>) : go(&phiT_contract_kernel<DH, 32, false, D64, D64>);
  } else if (deep) {
    if (wide) orows ? go(&phiT_contract_kernel<DH, FWB, true, false, D64>) : go(&phiT_contract_kernel<DH, FWB, false, false, D64>);
    else orows ? go(&phiT_contract_kernel<DH, 32, true, false, D64>) : go(&phiT_contract_kernel<DH, 32, false, false, D64>);
  } else if (wide) {
    if (orows) ragged ? go(&phiT_contract_kernel<DH, FWB, true, true, false>) : go(&phiT_contract_kernel<DH, FWB, true, false, false>);
    else ragged ? go(&phiT_contract_kernel<DH, FWB, false, true, false>) : go(&phiT_contract_kernel<DH, FWB, false, false, false>);
  } else {
    if (orows) ragged ? go(&phiT_contract_kernel<DH, 32, true, true, false>) : go(&phiT_contract_kernel<DH, 32, true, false, false>);
    else ragged ? go(&phiT_contract_kernel<DH, 32, false, true, false>) : go(&phiT_contract_kernel<DH, 32, false, false, false>);
  }
  const int64_t W = (int64_t)c.m * DH;
  WERSA_STAGE("wersa_reduce_contract", st,
              reduce_contract_kernel<DH><<<dim3((unsigned)(W / 64 + c.m / 64), slices), 256, 0, st>>>(
                  w.Spart, w.zpart, p.chunksC, c.m, w.coef + kCoefCscale, S, z, Mx, MT, bb));
}

template <int DH>
wersa_status fast_forward_t(const wersa_desc &c, const bf16_t *q, const bf16_t *k, const bf16_t *v,
                            const bf16_t *omega, const float *sigma, const float *gate_w,
                            const float *gate_b, const float *scale_w, bf16_t *out, float *saved,
                            float *ws, hipStream_t st, const PooledSums *pooled) {
  const FastPlan p = fast_plan(c);
  const FastWs w = fast_ws(c, p, 0, ws, saved);
  const SavedLayout sv = saved_layout(c);
  const int slices = c.B * c.H;
  const View tv{c.stride_b, c.stride_h, c.stride_n, c.H};
  float *S = saved + sv.S, *z = saved + sv.z, *qbar = saved + sv.qbar, *s = saved + sv.s,
        *F = saved + sv.F, *D = saved + sv.D;
  _Float16 *QF = sv.QF >= 0 ? reinterpret_cast<_Float16 *>(saved + sv.QF) : nullptr;
  _Float16 *KF = sv.KF >= 0 ? reinterpret_cast<_Float16 *>(saved + sv.KF) : nullptr;

  const int nmat = (c.flags & WERSA_FLAG_SEPARATE_OMEGA) ? 2 : 1;
  SetupArgs su{sigma, c.bw_floor, omega, c.d, c.m, nmat, w.scalars, w.omT, setup_blocks(c.d, c.m, nmat)};
  const SetupArgs none{};
  const bool deep = c.L > kTileL;
  if (pooled && c.n % 128 == 0 && !deep) {
    WERSA_STAGE("wersa_setup", st, setup_kernel<<<su.blocks, 256, 0, st>>>(su));
    // the caller's column sums per 128 token rows: batch b owns row blocks [b n/128, (b+1) n/128)
    const int chunks = c.n / 128;
    WERSA_STAGE("gate_fwd_kernel", st,
                gate_fwd_kernel<<<slices, 256, 0, st>>>(pooled->sums, chunks, c.n, c.d, c.L, c.H, gate_w, gate_b, scale_w,
                                                       qbar, s, F, w.coef, (c.flags & WERSA_FLAG_POOLED_GATE) ? 1 : 0,
                                                       PooledLayout{chunks * pooled->hidden, c.d, pooled->hidden},
                                                       pooled->amax, chunks * (c.d / kPooledMaxCols), w.scalars,
                                                       AmaxLayout{chunks * (pooled->hidden / kPooledMaxCols), c.d / kPooledMaxCols,
                                                                  pooled->hidden / kPooledMaxCols, c.d / kPooledMaxCols}));
  } else {
    // deep: one partial per 64-row tile, kept (with those of K) as the tile sums of the levels above 6
    float *qpart = deep ? w.tileQ : w.qpart;
    WERSA_STAGE("wersa_qbar", st,
                qbar_partial_kernel<DH><<<dim3(p.chunksQ + su.blocks, slices), 256, 0, st>>>(q, tv, c.n, p.rowsQ, qpart,
                                                                                             p.chunksQ, su, w.qamax));
    WERSA_STAGE("gate_fwd_kernel", st,
                gate_fwd_kernel<<<slices, 256, 0, st>>>(qpart, p.chunksQ, c.n, c.d, c.L, c.H, gate_w, gate_b, scale_w,
                                                       qbar, s, F, w.coef, (c.flags & WERSA_FLAG_POOLED_GATE) ? 1 : 0,
                                                       PooledLayout{(int64_t)c.H * p.chunksQ * c.d, (int64_t)p.chunksQ * c.d, c.d},
                                                       w.qamax, p.chunksQ, w.scalars,
                                                       AmaxLayout{(int64_t)c.H * p.chunksQ, p.chunksQ, 0, p.chunksQ}));
  }
  if (deep) {
    WERSA_STAGE("wersa_qbar", st,
                qbar_partial_kernel<DH><<<dim3(p.chunksQ, slices), 256, 0, st>>>(k, tv, c.n, p.rowsQ, w.tileK,
                                                                                 p.chunksQ, none, nullptr));
    WERSA_STAGE("wersa_coarse_addend", st,
                coarse_addend_kernel<<<dim3(slices, 2, DH / kCoarseCols), 1024, 0, st>>>(w.tileQ, w.tileK, w.coef, p.chunksQ, DH, c.L, w.pyr,
                                                                      w.addQ, w.addK));
  }
  if (DH != 64) {   // head dimension 64 runs stage A inside the kernels that consume X_F
    WERSA_STAGE("wersa_haar_stage", st,
                haar_stage_kernel<DH><<<dim3((c.n + 63) / 64, slices), 256, 0, st>>>(q, tv, c.n, w.coef, deep ? w.addQ : nullptr, QF));
    WERSA_STAGE("wersa_haar_stage", st,
                haar_stage_kernel<DH><<<dim3((c.n + 63) / 64, slices), 256, 0, st>>>(k, tv, c.n, w.coef, deep ? w.addK : nullptr, KF));
  }
  launch_contract<DH>(c, p, KF, k, v, tv, nullptr, nullptr, nullptr, true, w, S, z, w.Sx, w.ST, w.zb, st);
  if (launch_rows<DH, 0>(c, p, QF, q, nullptr, nullptr, nullptr, w, omega, nullptr, w.ST, w.zb, out, D,
                         nullptr, st) != hipSuccess)
    return WERSA_ERR_LAUNCH;
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

template <int DH>
wersa_status fast_backward_t(const wersa_desc &c, const bf16_t *q, const bf16_t *k, const bf16_t *v,
                             const bf16_t *omega, const float *sigma, const float *gate_w,
                             const float *scale_w, const bf16_t *out, const bf16_t *dout,
                             const float *saved, bf16_t *dq, bf16_t *dk, bf16_t *dv, float *dgate_w,
                             float *dgate_b, float *dscale_w, float *dsigma, float *ws,
                             hipStream_t st) {
  const FastPlan p = fast_plan(c);
  const FastWs w = fast_ws(c, p, 1, ws, const_cast<float *>(saved));   // operand copies are only read
  const SavedLayout sv = saved_layout(c);
  const int slices = c.B * c.H;
  const View tv{c.stride_b, c.stride_h, c.stride_n, c.H};
  const float *qbar = saved + sv.qbar, *s = saved + sv.s, *D = saved + sv.D;
  const _Float16 *QF = sv.QF >= 0 ? reinterpret_cast<const _Float16 *>(saved + sv.QF) : nullptr;
  const _Float16 *KF = sv.KF >= 0 ? reinterpret_cast<const _Float16 *>(saved + sv.KF) : nullptr;

  // dS = Phi_Q^T dN, dz = Phi_Q^T dD; the same pass derives dD_t = -<dO_t, O_t> / D_t from the
  // rows of O and leaves it in the workspace for the Q-side gradient kernel.
  const bool ln = (c.flags & WERSA_FLAG_LAYERNORM) != 0;
  // LayerNorm output stage: dN first, then the same kernels with D = 1 and dD = 0 (so dz = 0).
  const View nv{(int64_t)c.H * c.n * DH, (int64_t)c.n * DH, DH, c.H};
  if (ln) {
    WERSA_STAGE("wersa_ln_prep", st,
                ln_prep_kernel<DH><<<dim3(p.chunksC, slices), 256, 0, st>>>(dout, out, tv, D, c.n, p.rowsC, w.dN,
                                                                           w.ones, w.dD, w.dDpart));
    launch_contract<DH>(c, p, QF, q, w.dN, nv, nullptr, w.dD, nullptr, false, w, w.dS, w.dz, w.dSx, w.dST, w.dzb, st);
  } else {
    launch_contract<DH>(c, p, QF, q, dout, tv, D, nullptr, out, false, w, w.dS, w.dz, w.dSx, w.dST, w.dzb, st);
  }
  // K side first: the Q-side kernel then is the last writer of a large tensor before the pass
  // that adds the pooled-query term to dQ, which finds part of dQ still in the last-level cache.
  const bool dv_too = dv_rides_along(c, p);
  if (launch_rows<DH, 2>(c, p, KF, k, v, nullptr, nullptr, w, omega, w.dSx, nullptr, nullptr, dk, nullptr,
                         w.partK, st, nullptr, dv_too ? dv : nullptr) != hipSuccess)
    return WERSA_ERR_LAUNCH;
  if (!dv_too && launch_rows<DH, 3>(c, p, KF, k, nullptr, nullptr, nullptr, w, omega, nullptr, w.dST, nullptr, dv,
                                    nullptr, nullptr, st) != hipSuccess)
    return WERSA_ERR_LAUNCH;
  if (ln) {
    if (launch_rows<DH, 1>(c, p, QF, q, w.dN, w.ones, w.dD, w, omega, w.Sx, nullptr, nullptr, dq, nullptr,
                           w.partQ, st, &nv) != hipSuccess)
      return WERSA_ERR_LAUNCH;
  } else {
    if (launch_rows<DH, 1>(c, p, QF, q, dout, D, w.dD, w, omega, w.Sx, nullptr, nullptr, dq, nullptr,
                           w.partQ, st) != hipSuccess)
      return WERSA_ERR_LAUNCH;
  }
  const bool deep = c.L > kTileL;
  if (deep)   // levels above 6: addends of dQ and dK and the bands' extra row, from the tile sums
    WERSA_STAGE("wersa_coarse_bwd", st,
                coarse_bwd_kernel<<<dim3(slices, 2, DH / kCoarseCols), 1024, 0, st>>>(w.gsumQ, w.gsumK, w.tileQ, w.tileK, w.coef,
                                                                   (c.n + 63) / 64, DH, c.L, w.pyr, w.gaddQ, w.gaddK,
                                                                   w.partQ, w.partK, p.rowsWgsG));
  WERSA_STAGE("gate_bwd_slice_kernel", st,
              gate_bwd_slice_kernel<<<slices, kGateBwdThreads, 0, st>>>(w.partQ, w.partK, deep ? p.rowsWgsG + DH / kCoarseCols : p.rowsWgsG, c.L,
                                                           c.d, c.H, s, gate_w, scale_w, w.dF, w.dlogit, w.dqbar,
                                                           (c.flags & WERSA_FLAG_POOLED_GATE) ? 1 : 0, w.coef));
  WERSA_STAGE("gate_bwd_params_kernel", st,
              gate_bwd_params_kernel<<<gate_bwd_params_blocks(c.H, c.L, c.d), 256, 0, st>>>(w.dF, w.dlogit, s, qbar, w.dDpart, slices * p.chunksC,
                                                        c.B, c.H, c.L, c.d, c.eps, w.scalars, dgate_w,
                                                        dgate_b, dscale_w, dsigma));
  const int64_t chunks = (int64_t)c.n * (DH / 8);
  const dim3 agrid((unsigned)((chunks + 1023) / 1024), slices);
  if (deep) {
    WERSA_STAGE("wersa_add_pooled", st,
                (add_pooled_kernel<DH, true><<<agrid, 256, 0, st>>>(dq, tv, w.dqbar, c.n, 1.0f / (float)c.n, w.gaddQ)));
    WERSA_STAGE("wersa_add_pooled", st,
                (add_pooled_kernel<DH, true><<<agrid, 256, 0, st>>>(dk, tv, nullptr, c.n, 0.f, w.gaddK)));
  } else {
    WERSA_STAGE("wersa_add_pooled", st,
                (add_pooled_kernel<DH, false><<<agrid, 256, 0, st>>>(dq, tv, w.dqbar, c.n, 1.0f / (float)c.n, nullptr)));
  }
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

}  // namespace

bool fast_haar_filter_supported(const wersa_desc &c, const void *x, const void *xf) {
  return c.dtype == WERSA_BF16 && c.L <= kTileL && c.d % 8 == 0 && c.stride_n % 8 == 0 && c.stride_h % 8 == 0 &&
         c.stride_b % 8 == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)xf % 16) == 0;
}

wersa_status fast_haar_filter(const wersa_desc &c, const void *x, const float *filt, void *xf, hipStream_t st) {
  const View tv{c.stride_b, c.stride_h, c.stride_n, c.H};
  const dim3 grid((unsigned)((c.n + 63) / 64), (unsigned)((c.d + 63) / 64), (unsigned)(c.B * c.H));
  WERSA_STAGE("wersa_haar_filter_bf16", st,
              haar_filter_bf16_kernel<<<grid, 256, 0, st>>>((const bf16_t *)x, (bf16_t *)xf, tv, c.n, c.d, filt, c.L));
  return hipGetLastError() == hipSuccess ? WERSA_OK : WERSA_ERR_LAUNCH;
}

bool fast_supported(const wersa_desc &c) {
  return c.dtype == WERSA_BF16 && (c.d == 64 || c.d == 128) && c.m % 128 == 0 &&
         c.stride_n % 8 == 0 && c.stride_h % 8 == 0 && c.stride_b % 8 == 0;
}

size_t fast_workspace_bytes(const wersa_desc &c, int for_backward) {
  return (size_t)fast_ws(c, fast_plan(c), for_backward, nullptr, nullptr).total * sizeof(float);
}

wersa_status fast_forward(const wersa_desc &c, const void *q, const void *k, const void *v,
                          const void *omega_rf, const float *sigma, const float *gate_w,
                          const float *gate_b, const float *scale_w, void *out, float *saved,
                          float *ws, hipStream_t st, const PooledSums *pooled) {
  if (c.d == 64)
    return fast_forward_t<64>(c, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                              (const bf16_t *)omega_rf, sigma, gate_w, gate_b, scale_w, (bf16_t *)out,
                              saved, ws, st, pooled);
  return fast_forward_t<128>(c, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                             (const bf16_t *)omega_rf, sigma, gate_w, gate_b, scale_w, (bf16_t *)out,
                             saved, ws, st, pooled);
}

wersa_status fast_backward(const wersa_desc &c, const void *q, const void *k, const void *v,
                           const void *omega_rf, const float *sigma, const float *gate_w,
                           const float *scale_w, const void *out, const void *dout,
                           const float *saved, void *dq, void *dk, void *dv, float *dgate_w,
                           float *dgate_b, float *dscale_w, float *dsigma, float *ws,
                           hipStream_t st) {
  if (c.d == 64)
    return fast_backward_t<64>(c, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                               (const bf16_t *)omega_rf, sigma, gate_w, scale_w, (const bf16_t *)out,
                               (const bf16_t *)dout, saved, (bf16_t *)dq, (bf16_t *)dk, (bf16_t *)dv,
                               dgate_w, dgate_b, dscale_w, dsigma, ws, st);
  return fast_backward_t<128>(c, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                              (const bf16_t *)omega_rf, sigma, gate_w, scale_w, (const bf16_t *)out,
                              (const bf16_t *)dout, saved, (bf16_t *)dq, (bf16_t *)dk, (bf16_t *)dv,
                              dgate_w, dgate_b, dscale_w, dsigma, ws, st);
}

}  // namespace wersa
