// Optional per-kernel timing with HIP events on the caller's stream (off by default).
// When enabled, every kernel launch of the library is bracketed by an event pair; reading
// the results synchronises those events.  Not thread-safe; meant for benchmarks and tools.
#include "wersa_internal.h"

#include <string.h>
#include <string>
#include <vector>

namespace wersa {
namespace {
struct Rec {
  const char *name;
  hipEvent_t a, b;
};
bool g_on = false;
bool g_open = false;        // the last prof_begin recorded an event pair
std::string g_only;         // when not empty: bracket only launches of this name
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
size_t g_pool_used = 0;
constexpr size_t kMaxEvents = 1 << 16;

hipEvent_t take_event() {
  if (g_pool_used == g_pool.size()) {
    if (g_pool.size() >= kMaxEvents) return nullptr;
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    g_pool.push_back(e);
  }
  return g_pool[g_pool_used++];
}
struct Agg {
  std::string name;
  double ms;
  int launches;
};
std::vector<Agg> g_agg;
}  // namespace

// ---- reference microbenchmarks: what this device sustains on a plain streaming copy and on a
// loop of independent matrix instructions, for roofline fractions against measured peaks --------
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 pk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f32x16 __attribute__((ext_vector_type(16)));

// dst[i] = src[i] for `pieces` 16-byte pieces: each workgroup streams contiguous runs of 8 x 4 KiB,
// eight independent 16-byte loads per thread in flight before the first store.
__global__ __launch_bounds__(256) void peak_copy_kernel(u32x4 *dst, const u32x4 *src, size_t pieces) {
  constexpr size_t RUN = 8 * 256;   // pieces per workgroup per round
  const size_t rounds = pieces / RUN;
  for (size_t r = blockIdx.x; r < rounds; r += gridDim.x) {
    const size_t i0 = r * RUN + threadIdx.x;
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i0 + 256 * u);
#pragma unroll
    for (int u = 0; u < 8; ++u) __builtin_nontemporal_store(v[u], dst + i0 + 256 * u);
  }
  if (blockIdx.x == 0)
    for (size_t i = rounds * RUN + threadIdx.x; i < pieces; i += 256) dst[i] = src[i];
}

// Every wave issues iters x 4 independent v_mfma_f32_32x32x16_bf16 (four accumulator tiles, operands
// in registers): no memory traffic, nothing but the matrix pipe.  The store never happens (the
// accumulators cannot reach that value); it keeps the loop alive.
__global__ __launch_bounds__(256) void peak_mfma_kernel(int iters, float seed, float *sink) {
  pk_bf16x8 a, b;
  for (int q = 0; q < 8; ++q) {
    a[q] = (__bf16)(seed + 0.001f * (float)(threadIdx.x + q));
    b[q] = (__bf16)(seed - 0.002f * (float)(threadIdx.x ^ q));
  }
  pk_f32x16 c0, c1, c2, c3;
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == -1.2345e30f) sink[0] = s;
}

bool profiling() { return g_on; }

void prof_begin(const char *name, hipStream_t st) {
  g_open = false;
  if (!g_on) return;
  if (!g_only.empty() && g_only != name) return;
  hipEvent_t a = take_event(), b = take_event();
  if (!a || !b) return;
  g_recs.push_back(Rec{name, a, b});
  (void)hipEventRecord(a, st);
  g_open = true;
}
void prof_end(hipStream_t st) {
  if (!g_on || !g_open || g_recs.empty()) return;
  (void)hipEventRecord(g_recs.back().b, st);
  g_open = false;
}
}  // namespace wersa

using namespace wersa;

extern "C" {

void wersa_profile_enable(int on) {
  g_on = on != 0;
}

void wersa_profile_only(const char *name) {
  g_only = name ? name : "";
}

void wersa_profile_reset(void) {
  g_recs.clear();
  g_agg.clear();
  g_pool_used = 0;
}

int32_t wersa_profile_collect(void) {
  g_agg.clear();
  for (const Rec &r : g_recs) {
    if (hipEventSynchronize(r.b) != hipSuccess) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) continue;
    bool found = false;
    for (Agg &a : g_agg)
      if (a.name == r.name) {
        a.ms += ms;
        a.launches += 1;
        found = true;
        break;
      }
    if (!found) g_agg.push_back(Agg{r.name, ms, 1});
  }
  g_recs.clear();
  g_pool_used = 0;
  return (int32_t)g_agg.size();
}

double wersa_peak_copy(void *dst, const void *src, size_t bytes, int32_t reps, void *hip_stream) {
  if (!dst || !src || bytes < 16 || reps < 1 || ((uintptr_t)dst % 16) || ((uintptr_t)src % 16)) return -1.0;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t pieces = bytes / 16;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return -1.0;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -1.0; }
  const unsigned grid = 256 * 8;   // eight workgroups of 256 threads per compute unit, each walking many rounds
  peak_copy_kernel<<<grid, 256, 0, st>>>((u32x4 *)dst, (const u32x4 *)src, pieces);   // warm-up
  (void)hipEventRecord(e0, st);
  for (int r = 0; r < reps; ++r) peak_copy_kernel<<<grid, 256, 0, st>>>((u32x4 *)dst, (const u32x4 *)src, pieces);
  (void)hipEventRecord(e1, st);
  float ms = 0.f;
  const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess &&
                  hipGetLastError() == hipSuccess && ms > 0.f;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return ok ? 2.0 * (double)(pieces * 16) * reps / (ms * 1e-3) / 1e9 : -1.0;
}

double wersa_peak_mfma(float *sink, int32_t reps, void *hip_stream) {
  if (!sink || reps < 1) return -1.0;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return -1.0;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -1.0; }
  const int blocks = 2048, iters = 4096;   // 8 waves per compute unit (two per SIMD), 16384 matrix instructions each
  peak_mfma_kernel<<<blocks, 256, 0, st>>>(64, 0.5f, sink);   // warm-up
  (void)hipEventRecord(e0, st);
  for (int r = 0; r < reps; ++r) peak_mfma_kernel<<<blocks, 256, 0, st>>>(iters, 0.5f, sink);
  (void)hipEventRecord(e1, st);
  float ms = 0.f;
  const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess &&
                  hipGetLastError() == hipSuccess && ms > 0.f;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  const double flop = (double)blocks * 4.0 * iters * 4.0 * (2.0 * 32 * 32 * 16) * reps;
  return ok ? flop / (ms * 1e-3) / 1e12 : -1.0;
}

int32_t wersa_profile_get(int32_t index, char *name, int32_t name_len, double *total_ms,
                          int32_t *launches) {
  if (index < 0 || index >= (int32_t)g_agg.size() || !name || name_len < 1 || !total_ms || !launches)
    return 1;
  strncpy(name, g_agg[index].name.c_str(), (size_t)name_len - 1);
  name[name_len - 1] = 0;
  *total_ms = g_agg[index].ms;
  *launches = g_agg[index].launches;
  return 0;
}

}  // extern "C"
