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

// Model of the forward tile kernel's inner loop with everything but its three pipes taken away: per
// MFMA one fresh 1 KiB A fragment from LDS (128-bit reads, the K tile's row stride) and the softmax
// arithmetic of one score per lane (fma, exp2, max, add, plus a conversion every other one), finely
// interleaved, two wavefronts per SIMD, pseudo-random operands; no global traffic, no barriers, no
// masks, no prologue or epilogue.  What it sustains is what this loop STRUCTURE can reach on the
// chip (it is power limited like the MFMA-only probe), a yardstick beside the data-sheet peak.
constexpr int MIX_LDS_BYTES = 65536;
__global__ __launch_bounds__(PROBE_THREADS) void mix_probe_kernel(float* __restrict__ out, int iters,
                                                                  unsigned long long* __restrict__ clocks) {
  extern __shared__ __attribute__((aligned(16))) char mix_lds[];
  const unsigned base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)mix_lds;
  const int tid = threadIdx.x, lane = tid & 63;
  // 64 KiB of pseudo-random bf16 of unit scale
  for (int i = tid; i < MIX_LDS_BYTES / 2; i += PROBE_THREADS) {
    unsigned h = (blockIdx.x * 32768u + i + 1) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    reinterpret_cast<unsigned short*>(mix_lds)[i] = (unsigned short)((h & 0x807Fu) | ((125u + ((h >> 9) & 3u)) << 7));
  }
  __syncthreads();
  bf16x8 q[8], a[4];
#pragma unroll
  for (int f = 0; f < 8; ++f) q[f] = lds_load_b128(base + ((lane * 16 + f * 1024 + (tid >> 6) * 8192) & (MIX_LDS_BYTES - 1)));
  f32x16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = zero16();
  float sv[16], mx = -1e30f, sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) sv[r] = (float)(lane + r) * 0.01f;
  // fragment reads like the K tile's: row (lane & 31) of 272 bytes, 16-byte half (lane >> 5); every
  // address below stays under 8448 + 32767 + 224 + 16 < 64 KiB
  const unsigned rd = base + (lane & 31) * 272 + (lane >> 5) * 16;
#pragma unroll
  for (int f = 0; f < 4; ++f) a[f] = lds_load_b128(rd + f * 32);
  const unsigned long long c0 = __builtin_readcyclecounter();
  const unsigned long long w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int x = 0; x < PROBE_MFMA_PER_ITER; ++x) {
      acc[x & 3] = mma(a[x & 3], q[x & 7], acc[x & 3]);
      a[x & 3] = lds_load_b128(rd + ((x * 32 + it * 8704) & 0x7FFF) + (x & 7) * 32);
      const float s = sv[x];
      mx = fmaxf(mx, s);
      const float p = fast_exp2(fmaf(s, 0.127f, -3.0f));
      sum += p;
      sv[x] = p * 1.001f + 0.5f;                  // keeps the chain alive and bounded
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA,
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read,
      __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);   // five vector-ALU instructions
    }
  }
  const unsigned long long c1 = __builtin_readcyclecounter();
  const unsigned long long w1 = wall_clock64();
  float r = sum + mx;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) r += acc[t][e];
#pragma unroll
  for (int e = 0; e < 16; ++e) r += sv[e];
  out[blockIdx.x * PROBE_THREADS + tid] = r;
  if (tid == 0 && blockIdx.x == 0) { clocks[0] = c1 - c0; clocks[1] = w1 - w0; }
}

// Model of the dK/dV kernel's inner loop, in the same spirit: eight wavefronts in four pairs (w, w + 4:
// one SIMD each).  Per step of 32 query rows a wavefront issues 8 MFMAs on fresh natural fragments
// (128-bit LDS reads, rows of 320 bytes), turns the 16 results per lane into the B operand of the
// second contraction - the score role by fma + exp2, handing its probabilities to the partner as
// fp32 through a 4 KiB LDS mailbox, the gradient role by multiplying with the partner's
// probabilities of the step before - and issues 8 MFMAs whose A fragments come from the LDS
// transpose read; one barrier per step.  Pseudo-random operands; no global traffic, masks,
// staging, statistics, dS hand-over, prologue or epilogue.
// LEAVE: parts of the model left out, to see what each costs - bit 0 the mailbox (the gradient
// role multiplies with constants), bit 1 the element-wise arithmetic (the first contraction's
// results are only rounded), bit 2 the barrier (only together with bit 0: without the barrier
// nothing may pass between wavefronts).
constexpr int BMIX_MBOX = MIX_LDS_BYTES;                       // mailboxes behind the 64 KiB of operands
constexpr int BMIX_LDS_BYTES = MIX_LDS_BYTES + 4 * 2 * 4096;   // four pairs x two slots x 4 KiB
template <int LEAVE>
__global__ __launch_bounds__(PROBE_THREADS) void bwd_mix_probe_kernel(float* __restrict__ out, int iters,
                                                                      unsigned long long* __restrict__ clocks) {
  static_assert(!(LEAVE & 4) || (LEAVE & 1), "no barrier only without the mailbox");
  extern __shared__ __attribute__((aligned(16))) char mix_lds[];
  const unsigned base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)mix_lds;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int role = wave >> 2, pair = wave & 3;
  for (int i = tid; i < MIX_LDS_BYTES / 2; i += PROBE_THREADS) {
    unsigned h = (blockIdx.x * 32768u + i + 1) * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    reinterpret_cast<unsigned short*>(mix_lds)[i] = (unsigned short)((h & 0x807Fu) | ((125u + ((h >> 9) & 3u)) << 7));
  }
  for (int i = tid; i < (BMIX_LDS_BYTES - MIX_LDS_BYTES) / 4; i += PROBE_THREADS)
    reinterpret_cast<float*>(mix_lds + BMIX_MBOX)[i] = 0.25f;
  __syncthreads();
  bf16x8 kf[8];                                   // the register-resident fragments (K^T or V^T)
#pragma unroll
  for (int f = 0; f < 8; ++f) kf[f] = lds_load_b128(base + ((lane * 16 + f * 1024 + wave * 8192) & (MIX_LDS_BYTES - 1)));
  f32x16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = zero16();
  // natural reads: row (lane & 31) of 320 bytes, 16-byte half (lane >> 5); transposing reads: the
  // 8-byte pieces of rows 4 * (g16 >> 1) + (j16 >> 2) and + 8.  Every address stays below
  // 32767 + 31 * 320 + 16 + 7 * 32 + 16 < 64 KiB.
  const int g16 = lane >> 4, j16 = lane & 15;
  const unsigned nat = base + (lane & 31) * 320 + (lane >> 5) * 16;
  const unsigned tr = base + (4 * (g16 >> 1) + (j16 >> 2)) * 320 + (16 * (g16 & 1) + 4 * (j16 & 3)) * 2;
  const unsigned mbox = base + BMIX_MBOX + pair * 8192 + lane * 16;
  const unsigned long long c0 = __builtin_readcyclecounter();
  const unsigned long long w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    const unsigned mv = (unsigned)(it * 2560) & 0x7FFF;       // the tiles move through the 64 KiB
    const unsigned slot = (it & 1) * 4096;
    bf16x8 a[4];
#pragma unroll
    for (int f = 0; f < 4; ++f) a[f] = lds_load_b128(nat + mv + f * 32);
    f32x4 pm[4];
    if (role == 1) {
#pragma unroll
      for (int g = 0; g < 4; ++g)
        pm[g] = (LEAVE & 1) ? f32x4{0.3f, 0.2f, 0.1f, 0.4f}
                            : *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(
                                  (uintptr_t)(mbox + (slot ^ 4096) + g * 1024));
    }
    f32x16 s0 = zero16(), s1 = zero16();
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      if (x & 1) s1 = mma(a[x & 3], kf[x], s1); else s0 = mma(a[x & 3], kf[x], s0);
      if (x + 4 < 8) a[x & 3] = lds_load_b128(nat + mv + (x + 4) * 32);
    }
    bf16x8 t[4];
#pragma unroll
    for (int ht = 0; ht < 4; ++ht) t[ht] = lds_load_tr(tr + mv + 64 * ht, tr + mv + 64 * ht + 8 * 320);
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = s0[r] + s1[r];
    if (role == 0) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 p4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = (LEAVE & 2) ? s[4 * g + e] : fast_exp2(fmaf(s[4 * g + e], 0.1f, -8.0f));
          s[4 * g + e] = p;
          p4[e] = p;
        }
        if (!(LEAVE & 1))
          *reinterpret_cast<__attribute__((address_space(3))) f32x4*>((uintptr_t)(mbox + slot + g * 1024)) = p4;
      }
    } else {
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) s[4 * g + e] = (LEAVE & 2) ? s[4 * g + e] : pm[g][e] * s[4 * g + e] * 0.01f;
    }
    bf16x8 bf[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) bf[u] = pack8(s, 8 * u);
#pragma unroll
    for (int ht = 0; ht < 4; ++ht) {
      acc[ht] = mma(t[ht], bf[0], acc[ht]);
      t[ht] = lds_load_tr(tr + mv + 64 * ht + 16 * 320, tr + mv + 64 * ht + 24 * 320);
    }
#pragma unroll
    for (int ht = 0; ht < 4; ++ht) acc[ht] = mma(t[ht], bf[1], acc[ht]);
    if (!(LEAVE & 4)) __syncthreads();
  }
  const unsigned long long c1 = __builtin_readcyclecounter();
  const unsigned long long w1 = wall_clock64();
  float r = 0.f;
#pragma unroll
  for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
    for (int e = 0; e < 16; ++e) r += acc[t4][e];
  out[blockIdx.x * PROBE_THREADS + tid] = r;
  if (tid == 0 && blockIdx.x == 0) { clocks[0] = c1 - c0; clocks[1] = w1 - w0; }
}

// What the LDS of a compute unit delivers to eight wavefronts that do nothing but read it, with the
// two kinds of fragment reads the tile kernels use: KIND 0 128-bit reads (rows of 272 bytes, the K
// tile's pattern), KIND 1 64-bit transposing reads (rows of 320 bytes, the V tile's pattern).  16 reads
// per wavefront and iteration; the values are folded into one word so that no read can be dropped.
template <int KIND>
__global__ __launch_bounds__(PROBE_THREADS) void lds_read_probe_kernel(float* __restrict__ out, int iters,
                                                                       unsigned long long* __restrict__ clocks) {
  extern __shared__ __attribute__((aligned(16))) char mix_lds[];
  const unsigned base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)mix_lds;
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < MIX_LDS_BYTES / 4; i += PROBE_THREADS) reinterpret_cast<unsigned*>(mix_lds)[i] = i * 2654435761u;
  __syncthreads();
  const int g16 = lane >> 4, j16 = lane & 15;
  // every address stays below 32767 + 31 * 272 + 16 + 15 * 32 + 16 (KIND 0) or
  // 32767 + 7 * 320 + 56 + 192 + 28 * 320 + 8 (KIND 1), both < 64 KiB
  const unsigned addr = KIND == 0 ? base + (lane & 31) * 272 + (lane >> 5) * 16
                                  : base + (4 * (g16 >> 1) + (j16 >> 2)) * 320 + (16 * (g16 & 1) + 4 * (j16 & 3)) * 2;
  u32x4 acc = {0, 0, 0, 0};
  const unsigned long long c0 = __builtin_readcyclecounter();
  const unsigned long long w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    const unsigned mv = (unsigned)(it * 2560) & 0x7FFF;
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      if (KIND == 0) {
        acc ^= __builtin_bit_cast(u32x4, lds_load_b128(addr + mv + x * 32));
      } else {
        const unsigned a = addr + mv + (x & 3) * 64 + (x >> 2) * 8 * 320;
        acc ^= __builtin_bit_cast(u32x4, lds_load_tr(a, a + 4 * 320));   // two 64-bit transposing reads
      }
    }
  }
  const unsigned long long c1 = __builtin_readcyclecounter();
  const unsigned long long w1 = wall_clock64();
  out[blockIdx.x * PROBE_THREADS + tid] = __builtin_bit_cast(float, (acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) & 0x3FFFFFFFu);
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

// one workgroup per compute unit (64 KiB of LDS each); scratch as for launch_mfma_probe
hipError_t launch_mix_probe(int blocks, int iters, float* scratch, hipStream_t s) {
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(mix_probe_kernel), MIX_LDS_BYTES);
  if (e != hipSuccess) return e;
  unsigned long long* clocks = reinterpret_cast<unsigned long long*>(scratch + (size_t)blocks * PROBE_THREADS);
  hipLaunchKernelGGL(mix_probe_kernel, dim3(blocks), dim3(PROBE_THREADS), MIX_LDS_BYTES, s, scratch, iters, clocks);
  return hipGetLastError();
}

// one workgroup per compute unit (96 KiB of LDS each); scratch as for launch_mfma_probe;
// leave_out: 0, 1, 2, 3, 5 or 7 (the kernel's LEAVE)
namespace {
template <int LEAVE>
hipError_t bwd_mix_launch(int blocks, int iters, float* scratch, hipStream_t s) {
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(bwd_mix_probe_kernel<LEAVE>), BMIX_LDS_BYTES);
  if (e != hipSuccess) return e;
  unsigned long long* clocks = reinterpret_cast<unsigned long long*>(scratch + (size_t)blocks * PROBE_THREADS);
  hipLaunchKernelGGL(bwd_mix_probe_kernel<LEAVE>, dim3(blocks), dim3(PROBE_THREADS), BMIX_LDS_BYTES, s, scratch, iters,
                     clocks);
  return hipGetLastError();
}
template <int KIND>
hipError_t lds_read_launch(int blocks, int iters, float* scratch, hipStream_t s) {
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(lds_read_probe_kernel<KIND>), MIX_LDS_BYTES);
  if (e != hipSuccess) return e;
  unsigned long long* clocks = reinterpret_cast<unsigned long long*>(scratch + (size_t)blocks * PROBE_THREADS);
  hipLaunchKernelGGL(lds_read_probe_kernel<KIND>, dim3(blocks), dim3(PROBE_THREADS), MIX_LDS_BYTES, s, scratch, iters,
                     clocks);
  return hipGetLastError();
}
}  // namespace
hipError_t launch_bwd_mix_probe(int blocks, int iters, int leave_out, float* scratch, hipStream_t s) {
  switch (leave_out) {
    case 0: return bwd_mix_launch<0>(blocks, iters, scratch, s);
    case 1: return bwd_mix_launch<1>(blocks, iters, scratch, s);
    case 2: return bwd_mix_launch<2>(blocks, iters, scratch, s);
    case 3: return bwd_mix_launch<3>(blocks, iters, scratch, s);
    case 5: return bwd_mix_launch<5>(blocks, iters, scratch, s);
    case 7: return bwd_mix_launch<7>(blocks, iters, scratch, s);
    default: return hipErrorInvalidValue;
  }
}
// one workgroup of eight wavefronts per compute unit; kind 0: 128-bit reads, 1: transposing 64-bit reads
hipError_t launch_lds_read_probe(int blocks, int iters, int kind, float* scratch, hipStream_t s) {
  return kind == 0 ? lds_read_launch<0>(blocks, iters, scratch, s) : lds_read_launch<1>(blocks, iters, scratch, s);
}

int mfma_probe_threads() { return PROBE_THREADS; }
int mfma_probe_mfma_per_iter() { return PROBE_MFMA_PER_ITER; }

}  // namespace a2d
