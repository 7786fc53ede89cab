// Diagnostic: what the bf16 MFMA pipes of this chip sustain on their own, for pricing the
// tile kernels.  Wavefronts (at least two per SIMD: a single one can only issue an MFMA every
// other slot of the pipe) issue v_mfma_f32_32x32x16_bf16 back to back onto four independent
// accumulators with register operands - no LDS, no global traffic, no other arithmetic.  The result depends
// on the operand values: with random data the chip is power limited and lowers its clock, with
// constant data it is not, so both are measured.
#include <cstdio>

#include "a2d_common.hpp"
#include "a2d_mfma.hpp"

namespace a2d {
namespace {

using namespace mfma;

constexpr int PROBE_THREADS = 512;
constexpr int PROBE_MFMA_PER_ITER = 16;

__global__ __launch_bounds__(PROBE_THREADS) void mfma_probe_kernel(float* __restrict__ out, int iters,
                                                                   int random_data,
                                                                   unsigned long long* __restrict__ clocks) {
  const int tid = threadIdx.x;
  bf16x8 a[4], b;
  // pseudo-random values of roughly unit scale (sign, 7 mantissa bits, exponent 2^-2 .. 2^1), or 0.5
#pragma unroll
  for (int f = 0; f < 5; ++f)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      unsigned h = ((blockIdx.x * PROBE_THREADS + tid) * 40 + f * 8 + e + 1) * 2654435761u;
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
      const unsigned short bits =
          random_data ? (unsigned short)((h & 0x807Fu) | ((125u + ((h >> 9) & 3u)) << 7)) : (unsigned short)0x3F00u;
      const bf16_t v = __builtin_bit_cast(bf16_t, bits);
      if (f < 4) a[f][e] = v; else b[e] = v;
    }
  f32x16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = zero16();
  const unsigned long long c0 = __builtin_readcyclecounter();   // shader clock
  const unsigned long long w0 = wall_clock64();                  // constant 100 MHz
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int x = 0; x < PROBE_MFMA_PER_ITER; ++x) acc[x & 3] = mma(a[x & 3], b, acc[x & 3]);
  }
  const unsigned long long c1 = __builtin_readcyclecounter();
  const unsigned long long w1 = wall_clock64();
  float r = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int q = 0; q < 16; ++q) r += acc[t][q];
  out[blockIdx.x * PROBE_THREADS + tid] = r;
  if (tid == 0 && blockIdx.x == 0) { clocks[0] = c1 - c0; clocks[1] = w1 - w0; }
}

// Plain copy: every thread moves 16-byte pieces one grid-sized stride apart, four loads in flight.
__global__ __launch_bounds__(256) void copy_probe_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                         size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
    const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
    __builtin_nontemporal_store(a, dst + i);
    __builtin_nontemporal_store(b, dst + i + stride);
    __builtin_nontemporal_store(c, dst + i + 2 * stride);
    __builtin_nontemporal_store(d, dst + i + 3 * stride);
  }
  for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

hipError_t launch_copy_probe(void* dst, const void* src, size_t n16, hipStream_t s) {
  int cus = 0;
  const hipError_t e = device_cus(&cus);
  if (e != hipSuccess) return e;
  // eight workgroups per compute unit, each thread walking the buffer in grid-sized strides
  const size_t want = (n16 + 255) / 256;
  const unsigned blocks = (unsigned)(want < (size_t)cus * 8 ? (want ? want : 1) : (size_t)cus * 8);
  hipLaunchKernelGGL(copy_probe_kernel, dim3(blocks), dim3(256), 0, s, (u32x4*)dst, (const u32x4*)src, n16);
  return hipGetLastError();
}

// scratch: (blocks * PROBE_THREADS) floats of results followed by two 64-bit counters
hipError_t launch_mfma_probe(int blocks, int iters, int random_data, float* scratch, hipStream_t s) {
  unsigned long long* clocks = reinterpret_cast<unsigned long long*>(scratch + (size_t)blocks * PROBE_THREADS);
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(PROBE_THREADS), 0, s, scratch, iters, random_data, clocks);
  return hipGetLastError();
}

int mfma_probe_threads() { return PROBE_THREADS; }
int mfma_probe_mfma_per_iter() { return PROBE_MFMA_PER_ITER; }

}  // namespace a2d
