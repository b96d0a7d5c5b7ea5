// Measured peaks of the machine, for the roofline figures of the benchmark (not part of the verification path, and not
// part of libspiffy.so: this file is a library of its own, libspiffy_probe.so, that only bench.py and one test load):
// a register-only loop of v_mfma_f32_32x32x16_bf16 on every SIMD, and a read-only stream over a device buffer.
#include "common.h"
#include "../../include/spiffy_probe.h"

namespace spiffy {

namespace {

constexpr int kProbeWgs = 1024;      // four workgroups of four wavefronts per CU: one wavefront per SIMD at a time is enough
constexpr int kChains = 4;           // independent accumulator chains per wavefront (hide the MFMA latency)

// every wavefront issues iters * kChains MFMAs; operands live in registers, nothing touches memory until the end
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int random_operands, float* __restrict__ sink) {
  bf16x8 a[kChains], b[kChains];
  f32x16 acc[kChains];
  unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int c = 0; c < kChains; ++c) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      // random operands: values in (-1, 1) that differ between lanes, elements and chains, so that consecutive
      // MFMAs see different bits; zero operands: the same instruction stream without the switching activity
      h = h * 1664525u + 1013904223u;
      const float x = random_operands ? ((float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f) : 0.f;
      h = h * 1664525u + 1013904223u;
      const float y = random_operands ? ((float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f) : 0.f;
      a[c][e] = static_cast<bf16_t>(x);
      b[c][e] = static_cast<bf16_t>(y);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
  }
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], b[c], acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[c][v];
  if (threadIdx.x == 0) sink[blockIdx.x] = s;
}

// every workgroup reads its contiguous share of the buffer, 16 bytes per lane and load, eight loads in flight per lane
__global__ __launch_bounds__(256) void probe_hbm_read_kernel(const uint4* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
  unsigned x = 0;
  size_t i = lo + threadIdx.x;
  for (; i + 7 * 256 < hi; i += 8 * 256) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + (size_t)u * 256];
#pragma unroll
    for (int u = 0; u < 8; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < hi; i += 256) {
    const uint4 v = src[i];
    x ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (x == 0x9e3779b9u) sink[0] = x;       // keeps the loads alive; practically never true
}

double probe_mfma_flop(int iters) { return (double)kProbeWgs * 4.0 * (double)iters * kChains * 2.0 * 32 * 32 * 16; }

}  // namespace

}  // namespace spiffy

extern "C" {
#pragma GCC visibility push(default)

int spiffy_probe_mfma(int32_t iters, int32_t random_operands, float* sink, double* flop, void* stream) {
  if (iters < 1 || iters > (1 << 24) || !sink || !flop) return SPIFFY_EINVAL;
  *flop = spiffy::probe_mfma_flop(iters);
  spiffy::probe_mfma_kernel<<<spiffy::kProbeWgs, 256, 0, (hipStream_t)stream>>>(iters, random_operands ? 1 : 0, sink);
  return hipGetLastError() == hipSuccess ? SPIFFY_OK : SPIFFY_EDEVICE;
}

int spiffy_probe_hbm_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
  if (!src || !sink || bytes < 16) return SPIFFY_EINVAL;
  if (reinterpret_cast<uintptr_t>(src) & 15u) return SPIFFY_EALIGN;
  spiffy::probe_hbm_read_kernel<<<2048, 256, 0, (hipStream_t)stream>>>(reinterpret_cast<const uint4*>(src), bytes / 16, sink);
  return hipGetLastError() == hipSuccess ? SPIFFY_OK : SPIFFY_EDEVICE;
}

#pragma GCC visibility pop
}  // extern "C"
