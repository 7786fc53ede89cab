// bf16 MFMA forward tile kernel for H = 128 (Sec. 3.1, Eq. (3), evaluated block by
// block with the recurrence of Sec. 2.2).
//
// Work split: one workgroup = 4 wavefronts = 128 query rows of one head; each
// wavefront owns 32 query rows for the whole kernel and walks the key blocks
// (64 keys per step) that the workgroup stages through LDS.
//
// Both contractions are issued TRANSPOSED so that no cross-lane data movement is
// needed between them (v_mfma_f32_32x32x16_bf16, D = A * B, A: 32 x 16, B: 16 x 32):
//   S^T = K * Q^T : A = K fragment (LDS, 128-bit reads), B = Q^T fragment (registers,
//                   loaded once).  In D a lane holds 16 keys of ONE query column, so
//                   row max / row sum are in-lane reductions plus one exchange with
//                   lane ^ 32.
//   O^T += V^T * P^T : B = P^T is exactly the D layout of S^T (the contraction index
//                   may be permuted freely as long as A uses the same permutation),
//                   A = V^T fragment read from the row-major V tile with the LDS
//                   transpose read ds_read_b64_tr_b16.
// LDS: K and V tiles double-buffered in the swizzled layout of a2d_mfma.hpp, which
// keeps both the 128-bit K reads and the transposing V reads bank-conflict free.
#include "a2d_mfma.hpp"

namespace a2d {
namespace {

using namespace mfma;

constexpr int BM = 128;            // query rows per workgroup
constexpr int BN = 64;             // keys per step
constexpr int kThreads = 256;
constexpr int kLdsBytes = 4 * TILE64_BYTES;   // K, V x two buffers

__global__ __launch_bounds__(kThreads, 2) void fwd_mfma_kernel(
    a2d_tile_desc d, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, float* __restrict__ O_part, float* __restrict__ m_out,
    float* __restrict__ l_out) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  // [buf] K tile at buf * 2 * TILE64_BYTES, V tile right after it

  const int head = blockIdx.y;
  // heavy (late) query blocks first: under a causal mask they walk more key blocks
  const int qb = gridDim.x - 1 - blockIdx.x;
  const int q0 = qb * BM;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int half = lane >> 5, l32 = lane & 31;
  Q += (int64_t)head * d.nq * H;
  K += (int64_t)head * d.nkv * H;
  V += (int64_t)head * d.nkv * H;
  FragAddr fa;
  fa.init(lane);

  // ---- Q^T fragments: lane holds query row (l32), h = 16*step + 8*half + 0..7
  const int q_row = q0 + wave * 32 + l32;
  bf16x8 qf[8];
  {
    const bool ok = q_row < d.nq;
    const bf16_t* qp = Q + (int64_t)(ok ? q_row : 0) * H + 8 * half;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      u32x4 w = *reinterpret_cast<const u32x4*>(qp + 16 * st);
      if (!ok) w = u32x4{0, 0, 0, 0};
      qf[st] = __builtin_bit_cast(bf16x8, w);
    }
  }

  // ---- visibility bounds in local key indices: query i sees key r iff r <= i + rel
  const int64_t rel = d.q_off - d.kv_off;
  auto vis_count = [&](int i) -> int {      // number of leading keys query row i can see
    if (!d.causal) return d.nkv;
    const int64_t v = (int64_t)i + rel + 1;
    return v <= 0 ? 0 : (v < d.nkv ? (int)v : d.nkv);
  };
  const int blk_last = min(q0 + BM, d.nq) - 1;
  const int nblk = (vis_count(blk_last) + BN - 1) / BN;
  const int w_first = q0 + wave * 32;
  const int w_last = min(w_first + 31, d.nq - 1);
  const int nvis_wave = (w_first < d.nq) ? vis_count(w_last) : 0;     // keys any row of the wave sees
  const int nfull_wave = (w_first < d.nq) ? vis_count(w_first) : 0;   // keys every row of the wave sees
  const int my_vis = (q_row < d.nq) ? vis_count(q_row) : 0;

  f32x16 o[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) o[t] = zero16();
  float m_run = -INFINITY;   // running max of the RAW dot products (scale applied on output)
  float l_run = 0.f;         // this lane's share of the running row sum
  const float c = d.scale * kLog2e;

  Stage64 kst, vst;
  if (nblk > 0) {
    kst.load(K, 0, d.nkv, tid);
    vst.load(V, 0, d.nkv, tid);
    kst.store(lds, tid);
    vst.store(lds + TILE64_BYTES, tid);
  }
  __syncthreads();

  for (int j = 0; j < nblk; ++j) {
    const int k0 = j * BN;
    const char* ks = lds + (j & 1) * 2 * TILE64_BYTES;
    const char* vs = ks + TILE64_BYTES;
    if (j + 1 < nblk) {
      kst.load(K, k0 + BN, d.nkv, tid);
      vst.load(V, k0 + BN, d.nkv, tid);
    }

    if (k0 < nvis_wave) {
      f32x16 s[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        s[t] = zero16();
#pragma unroll
        for (int st = 0; st < 8; ++st) s[t] = mma(read_nat(ks, fa, 32 * t, st), qf[st], s[t]);
      }
      // mask (only blocks that straddle the diagonal or the end of the tile)
      if (k0 + BN > nfull_wave) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + 32 * t + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key >= my_vis) s[t][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = fast_exp2((m_run - m_use) * c);
      const float mc = m_use * c;
      float psum = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = fast_exp2(fmaf(s[t][r], c, -mc));
          s[t][r] = p;
          psum += p;
        }
      l_run = fmaf(l_run, alpha, psum);
      m_run = m_new;
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] *= alpha;

#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bf16x8 pb = pack8(s[u >> 1], 8 * (u & 1));
#pragma unroll
        for (int ht = 0; ht < 4; ++ht) o[ht] = mma(read_tr(vs, fa, 16 * u, ht), pb, o[ht]);
      }
    }
    if (j + 1 < nblk) {
      char* nk = lds + ((j + 1) & 1) * 2 * TILE64_BYTES;
      kst.store(nk, tid);
      vst.store(nk + TILE64_BYTES, tid);
    }
    __syncthreads();
  }

  // ---- epilogue: N (unnormalised), m (scaled units), l
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (q_row < d.nq) {
    const int64_t row = (int64_t)head * d.nq + q_row;
    float* op = O_part + row * H + 4 * half;
#pragma unroll
    for (int ht = 0; ht < 4; ++ht)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 v = {o[ht][4 * g], o[ht][4 * g + 1], o[ht][4 * g + 2], o[ht][4 * g + 3]};
        *reinterpret_cast<f32x4*>(op + 32 * ht + 8 * g) = v;
      }
    if (half == 0) {
      m_out[row] = m_run * d.scale;   // -inf stays -inf (scale > 0)
      l_out[row] = l_tot;
    }
  }
}

}  // namespace

bool fwd_mfma_supported(const a2d_tile_desc& d) {
  return d.dtype == A2D_BF16 && d.hdim == mfma::H;
}

hipError_t launch_fwd_mfma(const a2d_tile_desc& d, const void* Q, const void* K, const void* V,
                           float* O_part, float* m, float* l, hipStream_t s) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fwd_mfma_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  if (e != hipSuccess) return e;
  dim3 grid((d.nq + BM - 1) / BM, d.heads), block(kThreads);
  hipLaunchKernelGGL(fwd_mfma_kernel, grid, block, kLdsBytes, s, d, (const bf16_t*)Q, (const bf16_t*)K,
                     (const bf16_t*)V, O_part, m, l);
  return hipGetLastError();
}

}  // namespace a2d
