// AttnFix (Alg. 2) folded over k partials + normalisation (Alg. 1 line 6), and the
// plain-sum merge of gradient partials (Alg. 3 lines 4-5).  Both are pure
// streaming kernels bound by HBM bandwidth: every input byte is read once with
// 128-bit loads, all k loads of a thread are issued before the first use.
#include "a2d_common.hpp"

namespace a2d {
namespace {

__device__ __forceinline__ void store_out4(float* O, int64_t off, f32x4 v) {
  *reinterpret_cast<f32x4*>(O + off) = v;
}
__device__ __forceinline__ void store_out4(bf16_t* O, int64_t off, f32x4 v) {
  bf16x4 b;
  b[0] = (bf16_t)v[0]; b[1] = (bf16_t)v[1]; b[2] = (bf16_t)v[2]; b[3] = (bf16_t)v[3];
  *reinterpret_cast<bf16x4*>(O + off) = b;
}

// One thread owns 4 consecutive columns of one row.  HV = H / 4 threads per row.
// KMAX is the unroll bound (k <= KMAX); loads of absent partials are predicated off.
template <typename OutT, int KMAX>
__global__ __launch_bounds__(256) void fix_kernel(FixPtrs p, int k, int64_t rows, int hv,
                                                  OutT* __restrict__ O, float* __restrict__ lse) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = idx / hv;
  const int c = (int)(idx - row * hv);
  if (row >= rows) return;
  const int64_t off = (row * hv + c) * 4;

  f32x4 n[KMAX];
  float mk[KMAX], lk[KMAX];
#pragma unroll
  for (int x = 0; x < KMAX; ++x) {
    if (x < k) {
      n[x] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p.o[x] + off));
      mk[x] = p.m[x][row];
      lk[x] = p.l[x][row];
    } else {
      n[x] = f32x4{0.f, 0.f, 0.f, 0.f};
      mk[x] = -INFINITY;
      lk[x] = 0.f;
    }
  }
  float M = -INFINITY;
#pragma unroll
  for (int x = 0; x < KMAX; ++x) M = fmaxf(M, mk[x]);
  float D = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int x = 0; x < KMAX; ++x) {
    // weight of partial x: exp(m_x - M); an empty partial (m = -inf) weighs 0
    const float w = (mk[x] == -INFINITY) ? 0.f : fast_exp2((mk[x] - M) * kLog2e);
    D = fmaf(w, lk[x], D);
    acc[0] = fmaf(w, n[x][0], acc[0]);
    acc[1] = fmaf(w, n[x][1], acc[1]);
    acc[2] = fmaf(w, n[x][2], acc[2]);
    acc[3] = fmaf(w, n[x][3], acc[3]);
  }
  const float inv = (D > 0.f) ? 1.0f / D : 0.f;
  acc[0] *= inv; acc[1] *= inv; acc[2] *= inv; acc[3] *= inv;
  store_out4(O, off, acc);
  if (c == 0) lse[row] = (D > 0.f) ? M + logf(D) : -INFINITY;
}

template <typename OutT, int KMAX>
__global__ __launch_bounds__(256) void sum_kernel(SumPtrs p, int k, int64_t n4,
                                                  OutT* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n4) return;
  f32x4 v[KMAX];
#pragma unroll
  for (int x = 0; x < KMAX; ++x) {
    if (x < k) v[x] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p.p[x]) + idx);
    else v[x] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  f32x4 acc = v[0];
#pragma unroll
  for (int x = 1; x < KMAX; ++x) {
    if (x < k) { acc[0] += v[x][0]; acc[1] += v[x][1]; acc[2] += v[x][2]; acc[3] += v[x][3]; }
  }
  store_out4(out, idx * 4, acc);
}

template <typename OutT>
hipError_t fix_dispatch(int k, int64_t rows, int hdim, const FixPtrs& p, OutT* O, float* lse,
                        hipStream_t s) {
  const int hv = hdim / 4;
  const int64_t threads = rows * hv;
  const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
  if (k <= 2) hipLaunchKernelGGL((fix_kernel<OutT, 2>), grid, block, 0, s, p, k, rows, hv, O, lse);
  else if (k <= 4) hipLaunchKernelGGL((fix_kernel<OutT, 4>), grid, block, 0, s, p, k, rows, hv, O, lse);
  else if (k <= 8) hipLaunchKernelGGL((fix_kernel<OutT, 8>), grid, block, 0, s, p, k, rows, hv, O, lse);
  else if (k <= 16) hipLaunchKernelGGL((fix_kernel<OutT, 16>), grid, block, 0, s, p, k, rows, hv, O, lse);
  else hipLaunchKernelGGL((fix_kernel<OutT, 32>), grid, block, 0, s, p, k, rows, hv, O, lse);
  return hipGetLastError();
}

template <typename OutT>
hipError_t sum_dispatch(int k, int64_t n, const SumPtrs& p, OutT* out, hipStream_t s) {
  const int64_t n4 = n / 4;
  const dim3 grid((unsigned)((n4 + 255) / 256)), block(256);
  if (k <= 2) hipLaunchKernelGGL((sum_kernel<OutT, 2>), grid, block, 0, s, p, k, n4, out);
  else if (k <= 4) hipLaunchKernelGGL((sum_kernel<OutT, 4>), grid, block, 0, s, p, k, n4, out);
  else if (k <= 8) hipLaunchKernelGGL((sum_kernel<OutT, 8>), grid, block, 0, s, p, k, n4, out);
  else if (k <= 16) hipLaunchKernelGGL((sum_kernel<OutT, 16>), grid, block, 0, s, p, k, n4, out);
  else hipLaunchKernelGGL((sum_kernel<OutT, 32>), grid, block, 0, s, p, k, n4, out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fix(int k, int64_t rows, int hdim, int out_dtype, const FixPtrs& p, void* O,
                      float* lse, hipStream_t s) {
  if (out_dtype == A2D_BF16) return fix_dispatch<bf16_t>(k, rows, hdim, p, (bf16_t*)O, lse, s);
  return fix_dispatch<float>(k, rows, hdim, p, (float*)O, lse, s);
}

hipError_t launch_fix_bwd(int k, int64_t n, int out_dtype, const SumPtrs& p, void* out,
                          hipStream_t s) {
  if (out_dtype == A2D_BF16) return sum_dispatch<bf16_t>(k, n, p, (bf16_t*)out, s);
  return sum_dispatch<float>(k, n, p, (float*)out, s);
}

}  // namespace a2d
