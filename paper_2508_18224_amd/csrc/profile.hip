// Optional per-kernel timing with HIP events on the caller's stream (see nsa_sel_profile_enable in nsa_sel.h).
#include <vector>

#include "common.h"

namespace nsa {
namespace {
struct Rec {
  int kid;
  hipEvent_t a, b;
};
std::vector<Rec> g_recs;
int g_used = 0;
bool g_on = false;
unsigned g_mask = ~0u;  // kernel kinds that are recorded (bit = index in kNames)
const char* const kNames[KID_COUNT] = {"index_prep", "index_chunk_prefix", "index_hist", "index_scan", "index_scatter",
                                       "index_finalize", "index_units", "fwd_main", "fwd_merge", "bwd_delta",
                                       "bwd_main", "bwd_dq_reduce", "bwd_dkv_reduce", "select_blocks", "fwd_query_outer",
                                       "index_dense", "fwd_dense"};
}  // namespace

ProfScope::ProfScope(int kid, hipStream_t stream) : slot(-1), st(stream) {
  if (!g_on || !((g_mask >> kid) & 1u) || g_used >= (int)g_recs.size()) return;
  slot = g_used++;
  g_recs[slot].kid = kid;
  (void)hipEventRecord(g_recs[slot].a, st);
}
ProfScope::~ProfScope() {
  if (slot >= 0) (void)hipEventRecord(g_recs[slot].b, st);
}
}  // namespace nsa

using namespace nsa;

// Plain streaming copy of 16-byte words: a kernel of known HBM traffic (bytes read + bytes written) against
// which hardware byte counters can be scaled.
__global__ void __launch_bounds__(256) k_calib_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

// Register-resident MFMA loop: every wavefront runs `iters` rounds of 8 independent v_mfma_f32_32x32x16_bf16
// chains (no memory traffic), so elapsed time gives the matrix-core rate this build can reach on the chip.
__global__ void __launch_bounds__(256) k_mfma_probe(int iters, float* __restrict__ sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (bf16_t)(0.001f * (float)(threadIdx.x + i));
    b[i] = (bf16_t)(0.002f * (float)(threadIdx.x ^ i));
  }
  f32x16 acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int c = 0; c < 8; ++c) t += acc[c][0];
  if (t == 12345.678f) sink[0] = t;  // keeps the loop alive
}

extern "C" {

int nsa_sel_mfma_probe(int iters, float* sink, double* flops, void* stream) {
  if (iters <= 0 || !sink) return NSA_SEL_EINVAL;
  const int blocks = 256 * 2;  // two 4-wave workgroups per CU
  hipLaunchKernelGGL(k_mfma_probe, dim3(blocks), dim3(256), 0, (hipStream_t)stream, iters, sink);
  if (flops) *flops = (double)blocks * 4.0 * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * 16.0;
  return hipGetLastError() == hipSuccess ? NSA_SEL_OK : NSA_SEL_EHIP;
}

int nsa_sel_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15) != 0) return NSA_SEL_EINVAL;
  if (bytes == 0) return NSA_SEL_OK;
  hipLaunchKernelGGL(k_calib_copy, dim3(256 * 32), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst,
                     bytes / 16);
  return hipGetLastError() == hipSuccess ? NSA_SEL_OK : NSA_SEL_EHIP;
}

int nsa_sel_profile_enable(int capacity) {
  for (auto& r : g_recs) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_recs.clear();
  g_used = 0;
  g_on = false;
  if (capacity <= 0) return NSA_SEL_OK;
  g_recs.resize(capacity);
  for (auto& r : g_recs) {
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return NSA_SEL_EHIP;
  }
  g_on = true;
  return NSA_SEL_OK;
}

int nsa_sel_profile_select(unsigned mask) {
  g_mask = mask;
  return NSA_SEL_OK;
}

int nsa_sel_profile_collect(int max_kernels, const char** names, float* total_ms, int* calls) {
  if (max_kernels < 0 || (max_kernels > 0 && (!names || !total_ms || !calls))) return NSA_SEL_EINVAL;
  const int n = max_kernels < KID_COUNT ? max_kernels : (int)KID_COUNT;
  for (int i = 0; i < n; ++i) {
    names[i] = kNames[i];
    total_ms[i] = 0.f;
    calls[i] = 0;
  }
  for (int i = 0; i < g_used; ++i) {
    float ms = 0.f;
    if (hipEventSynchronize(g_recs[i].b) != hipSuccess) return NSA_SEL_EHIP;
    if (hipEventElapsedTime(&ms, g_recs[i].a, g_recs[i].b) != hipSuccess) return NSA_SEL_EHIP;
    if (g_recs[i].kid < n) {
      total_ms[g_recs[i].kid] += ms;
      calls[g_recs[i].kid] += 1;
    }
  }
  g_used = 0;
  return n;
}

}  // extern "C"
