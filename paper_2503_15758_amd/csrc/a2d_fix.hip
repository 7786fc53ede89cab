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

// Where column group idx (4 columns, hv groups per row) of the merged output goes: plain, or row
// r of head h (nq rows per head) at h * head + r * row elements.
__device__ __forceinline__ int64_t out_offset(const OutMap& om, int64_t idx, int hv) {
  if (om.plain) return idx * 4;
  const int64_t row = idx / hv, h = row / om.nq;
  return h * om.head + (row - h * om.nq) * om.row + (idx - row * hv) * 4;
}

// Each thread handles CPT 16-byte column groups and issues the loads of all of them (CPT * k
// 128-bit loads) before the first use: the amount of data in flight per thread, not the
// arithmetic, decides how close these kernels get to the HBM rate (64 in flight cost occupancy
// and measured slower).
// (read once: non-temporal loads measured 8-10 % faster than plain ones here)
#define A2D_LD(p) __builtin_nontemporal_load(p)
constexpr int kLoadsInFlight = 32;
constexpr int chunks_per_thread(int kmax) { return kmax >= kLoadsInFlight ? 1 : kLoadsInFlight / kmax > 4 ? 4 : kLoadsInFlight / kmax; }
// (AttnFix carries m and l besides N: with 8 partials two chunks per thread - 16 loads of N in
// flight - leave room for more wavefronts and measured 3 % faster than four; 2, 4 and 16 partials
// are fastest with the common rule)
constexpr int chunks_per_thread_fix(int kmax) { return kmax == 8 ? 2 : chunks_per_thread(kmax); }

// Which column groups a thread owns: its wavefront owns CPT * 64 CONSECUTIVE groups and lane l takes
// the groups l, l + 64, ... of that run, so that every load instruction of a wavefront reads 1 KiB
// in one piece and its CPT loads of one partial read CPT KiB in one piece.  (Measured on MI355X: a
// read stream made of such per-wavefront runs of 4-16 KiB reaches 6.8-7.0 TB/s, the same bytes
// requested one grid-sized stride apart 5.3-6.4 TB/s.)
template <int CPT>
__device__ __forceinline__ int64_t group_index(int c) {
  const int64_t wave = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
  return wave * (CPT * 64) + c * 64 + (threadIdx.x & 63);
}

// A column group = 4 consecutive columns of one row; hv = H / 4 groups per row.
// KMAX is the unroll bound (k <= KMAX); loads of absent partials are predicated off.
// TRIPLE: the merge alone (Alg. 2 over k inputs): the result stays an unnormalised partial
// (N, m, l) - O receives N in fp32, lse receives m, l_out receives l.
template <typename OutT, int KMAX, int CPT, bool TRIPLE = false>
__global__ __launch_bounds__(256) void fix_kernel(FixPtrs p, int k, int64_t rows, int hv, OutMap om,
                                                  OutT* __restrict__ O, float* __restrict__ lse,
                                                  float* __restrict__ l_out) {
  const int64_t total = rows * hv;

  f32x4 n[CPT][KMAX];
  float mk[CPT][KMAX], lk[CPT][KMAX];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int64_t idx = group_index<CPT>(c);
    const int64_t row = idx / hv;
#pragma unroll
    for (int x = 0; x < KMAX; ++x) {
      if (x < k && idx < total) {
        n[c][x] = A2D_LD(reinterpret_cast<const f32x4*>(p.o[x]) + idx);
        mk[c][x] = p.m[x][row];
        lk[c][x] = p.l[x][row];
      } else {
        n[c][x] = f32x4{0.f, 0.f, 0.f, 0.f};
        mk[c][x] = -INFINITY;
        lk[c][x] = 0.f;
      }
    }
  }
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int64_t idx = group_index<CPT>(c);
    if (idx >= total) continue;
    const int64_t row = idx / hv;
    float M = -INFINITY;
#pragma unroll
    for (int x = 0; x < KMAX; ++x) M = fmaxf(M, mk[c][x]);
    float D = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int x = 0; x < KMAX; ++x) {
      // weight of partial x: exp(m_x - M); an empty partial (m = -inf) weighs 0
      const float w = (mk[c][x] == -INFINITY) ? 0.f : fast_exp2((mk[c][x] - M) * kLog2e);
      D = fmaf(w, lk[c][x], D);
      acc[0] = fmaf(w, n[c][x][0], acc[0]);
      acc[1] = fmaf(w, n[c][x][1], acc[1]);
      acc[2] = fmaf(w, n[c][x][2], acc[2]);
      acc[3] = fmaf(w, n[c][x][3], acc[3]);
    }
    if constexpr (TRIPLE) {
      store_out4(O, out_offset(om, idx, hv), acc);
      if (idx == row * hv) {
        lse[row] = M;
        l_out[row] = D;
      }
    } else {
      const float inv = (D > 0.f) ? 1.0f / D : 0.f;
      acc[0] *= inv; acc[1] *= inv; acc[2] *= inv; acc[3] *= inv;
      store_out4(O, out_offset(om, idx, hv), acc);
      if (idx == row * hv) lse[row] = (D > 0.f) ? M + logf(D) : -INFINITY;
    }
  }
}

template <typename OutT, int KMAX, int CPT>
__global__ __launch_bounds__(256) void sum_kernel(SumPtrs p, int k, int64_t n4, int hv, OutMap om,
                                                  OutT* __restrict__ out) {
  f32x4 v[CPT][KMAX];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int64_t idx = group_index<CPT>(c);
#pragma unroll
    for (int x = 0; x < KMAX; ++x) {
      if (x < k && idx < n4) v[c][x] = A2D_LD(reinterpret_cast<const f32x4*>(p.p[x]) + idx);
      else v[c][x] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int64_t idx = group_index<CPT>(c);
    if (idx >= n4) continue;
    // left-to-right sum over the partials (absent ones hold zeros)
    f32x4 acc = v[c][0];
#pragma unroll
    for (int x = 1; x < KMAX; ++x) {
      acc[0] += v[c][x][0]; acc[1] += v[c][x][1]; acc[2] += v[c][x][2]; acc[3] += v[c][x][3];
    }
    store_out4(out, out_offset(om, idx, hv), acc);
  }
}

// Merge of k NORMALISED partials: L = log sum_k exp(lse_k), O = sum_k exp(lse_k - L) O'_k.  A
// column group = 4 consecutive columns of one row, as in fix_kernel; InT is the partials' dtype.
template <typename InT, typename OutT, int KMAX, int CPT>
__global__ __launch_bounds__(256) void fix_norm_kernel(NormPtrs p, int k, int64_t rows, int hv, OutMap om,
                                                       OutT* __restrict__ O, float* __restrict__ lse) {
  const int64_t total = rows * hv;
  typedef InT in4 __attribute__((ext_vector_type(4)));
  in4 n[CPT][KMAX];
  float lk[CPT][KMAX];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int64_t idx = group_index<CPT>(c);
    const int64_t row = idx / hv;
#pragma unroll
    for (int x = 0; x < KMAX; ++x) {
      if (x < k && idx < total) {
        n[c][x] = A2D_LD(reinterpret_cast<const in4*>(p.o[x]) + idx);
        lk[c][x] = p.lse[x][row];
      } else {
        n[c][x] = in4{(InT)0.f, (InT)0.f, (InT)0.f, (InT)0.f};
        lk[c][x] = -INFINITY;
      }
    }
  }
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int64_t idx = group_index<CPT>(c);
    if (idx >= total) continue;
    const int64_t row = idx / hv;
    float M = -INFINITY;
#pragma unroll
    for (int x = 0; x < KMAX; ++x) M = fmaxf(M, lk[c][x]);
    float D = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int x = 0; x < KMAX; ++x) {
      // weight of partial x relative to the largest lse; an empty partial (lse = -inf) weighs 0
      const float w = (lk[c][x] == -INFINITY) ? 0.f : fast_exp2((lk[c][x] - M) * kLog2e);
      D += w;
      acc[0] = fmaf(w, to_f32(n[c][x][0]), acc[0]);
      acc[1] = fmaf(w, to_f32(n[c][x][1]), acc[1]);
      acc[2] = fmaf(w, to_f32(n[c][x][2]), acc[2]);
      acc[3] = fmaf(w, to_f32(n[c][x][3]), acc[3]);
    }
    const float inv = (D > 0.f) ? 1.0f / D : 0.f;
    acc[0] *= inv; acc[1] *= inv; acc[2] *= inv; acc[3] *= inv;
    store_out4(O, out_offset(om, idx, hv), acc);
    if (idx == row * hv) lse[row] = (D > 0.f) ? M + logf(D) : -INFINITY;
  }
}

template <typename OutT, int KMAX, bool TRIPLE = false>
void fix_launch(int k, int64_t rows, int hv, const FixPtrs& p, const OutMap& om, OutT* O, float* lse, float* l_out,
                hipStream_t s) {
  constexpr int CPT = chunks_per_thread_fix(KMAX);
  const int64_t per_block = 256 * CPT;
  const dim3 grid((unsigned)((rows * hv + per_block - 1) / per_block)), block(256);
  A2D_LAUNCH((fix_kernel<OutT, KMAX, CPT, TRIPLE>), grid, block, 0, s, p, k, rows, hv, om, O, lse, l_out);
}

template <typename OutT, int KMAX>
void sum_launch(int k, int64_t n4, int hv, const SumPtrs& p, const OutMap& om, OutT* out, hipStream_t s) {
  constexpr int CPT = chunks_per_thread(KMAX);
  const int64_t per_block = 256 * CPT;
  const dim3 grid((unsigned)((n4 + per_block - 1) / per_block)), block(256);
  A2D_LAUNCH((sum_kernel<OutT, KMAX, CPT>), grid, block, 0, s, p, k, n4, hv, om, out);
}

template <typename OutT, bool TRIPLE = false>
hipError_t fix_dispatch(int k, int64_t rows, int hdim, const FixPtrs& p, const OutMap& om, OutT* O, float* lse,
                        float* l_out, hipStream_t s) {
  const int hv = hdim / 4;
  if (k <= 2) fix_launch<OutT, 2, TRIPLE>(k, rows, hv, p, om, O, lse, l_out, s);
  else if (k <= 4) fix_launch<OutT, 4, TRIPLE>(k, rows, hv, p, om, O, lse, l_out, s);
  else if (k <= 8) fix_launch<OutT, 8, TRIPLE>(k, rows, hv, p, om, O, lse, l_out, s);
  else if (k <= 16) fix_launch<OutT, 16, TRIPLE>(k, rows, hv, p, om, O, lse, l_out, s);
  else fix_launch<OutT, 32, TRIPLE>(k, rows, hv, p, om, O, lse, l_out, s);
  return hipGetLastError();
}

template <typename OutT>
hipError_t sum_dispatch(int k, int64_t n, int hv, const SumPtrs& p, const OutMap& om, OutT* out, hipStream_t s) {
  const int64_t n4 = n / 4;
  if (k <= 2) sum_launch<OutT, 2>(k, n4, hv, p, om, out, s);
  else if (k <= 4) sum_launch<OutT, 4>(k, n4, hv, p, om, out, s);
  else if (k <= 8) sum_launch<OutT, 8>(k, n4, hv, p, om, out, s);
  else if (k <= 16) sum_launch<OutT, 16>(k, n4, hv, p, om, out, s);
  else sum_launch<OutT, 32>(k, n4, hv, p, om, out, s);
  return hipGetLastError();
}


template <typename InT, typename OutT, int KMAX>
void fix_norm_launch(int k, int64_t rows, int hv, const NormPtrs& p, const OutMap& om, OutT* O, float* lse, hipStream_t s) {
  constexpr int CPT = chunks_per_thread(KMAX);
  const int64_t per_block = 256 * CPT;
  const dim3 grid((unsigned)((rows * hv + per_block - 1) / per_block)), block(256);
  A2D_LAUNCH((fix_norm_kernel<InT, OutT, KMAX, CPT>), grid, block, 0, s, p, k, rows, hv, om, O, lse);
}

template <typename InT, typename OutT>
hipError_t fix_norm_dispatch(int k, int64_t rows, int hdim, const NormPtrs& p, const OutMap& om, OutT* O, float* lse,
                             hipStream_t s) {
  const int hv = hdim / 4;
  if (k <= 2) fix_norm_launch<InT, OutT, 2>(k, rows, hv, p, om, O, lse, s);
  else if (k <= 4) fix_norm_launch<InT, OutT, 4>(k, rows, hv, p, om, O, lse, s);
  else if (k <= 8) fix_norm_launch<InT, OutT, 8>(k, rows, hv, p, om, O, lse, s);
  else if (k <= 16) fix_norm_launch<InT, OutT, 16>(k, rows, hv, p, om, O, lse, s);
  else fix_norm_launch<InT, OutT, 32>(k, rows, hv, p, om, O, lse, s);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fix_norm(int k, int64_t rows, int hdim, int in_dtype, int out_dtype, const NormPtrs& p,
                           const OutMap& om, void* O, float* lse, hipStream_t s) {
  if (in_dtype == A2D_BF16) {
    if (out_dtype == A2D_BF16) return fix_norm_dispatch<bf16_t, bf16_t>(k, rows, hdim, p, om, (bf16_t*)O, lse, s);
    return fix_norm_dispatch<bf16_t, float>(k, rows, hdim, p, om, (float*)O, lse, s);
  }
  if (out_dtype == A2D_BF16) return fix_norm_dispatch<float, bf16_t>(k, rows, hdim, p, om, (bf16_t*)O, lse, s);
  return fix_norm_dispatch<float, float>(k, rows, hdim, p, om, (float*)O, lse, s);
}

hipError_t launch_fix(int k, int64_t rows, int hdim, int out_dtype, const FixPtrs& p, const OutMap& om, void* O,
                      float* lse, hipStream_t s) {
  if (out_dtype == A2D_BF16) return fix_dispatch<bf16_t>(k, rows, hdim, p, om, (bf16_t*)O, lse, nullptr, s);
  return fix_dispatch<float>(k, rows, hdim, p, om, (float*)O, lse, nullptr, s);
}

// the merge alone: k partials in, one unnormalised partial (N, m, l) out
hipError_t launch_attnfix(int k, int64_t rows, int hdim, const FixPtrs& p, float* N, float* m, float* l,
                          hipStream_t s) {
  return fix_dispatch<float, true>(k, rows, hdim, p, plain_out(), N, m, l, s);
}

// hv = column groups per row (only used when the output is not plain)
hipError_t launch_fix_bwd(int k, int64_t n, int hv, int out_dtype, const SumPtrs& p, const OutMap& om, void* out,
                          hipStream_t s) {
  if (out_dtype == A2D_BF16) return sum_dispatch<bf16_t>(k, n, hv, p, om, (bf16_t*)out, s);
  return sum_dispatch<float>(k, n, hv, p, om, (float*)out, s);
}

}  // namespace a2d
