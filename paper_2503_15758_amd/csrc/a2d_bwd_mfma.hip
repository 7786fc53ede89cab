// bf16 MFMA backward tile kernels for H = 128: the per-tile gradient call of Alg. 3
// line 3 with P = exp(S - lse) rebuilt from the FINAL log-sum-exp of the query block,
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Two kernels, so that every output has exactly one writer and no atomics are needed
// (bitwise reproducible results):
//   bwd_dkdv_kernel  owns key rows.   Workgroup = 128 keys (32 per wavefront, K and V
//                    fragments resident in registers); walks the query blocks, 64 rows
//                    per step, staged through LDS together with dO, lse and delta.
//                    S = Q K^T and dP = dO V^T leave a lane holding ONE key column, so
//                    P and dS feed dV^T += dO^T P and dK^T += Q^T dS directly as B
//                    operands; dO^T / Q^T come from the LDS transpose read.
//   bwd_dq_kernel    owns query rows. Workgroup = 128 queries (32 per wavefront, Q and
//                    dO fragments in registers); walks the key blocks, 64 keys per step.
//                    S^T = K Q^T and dP^T = V dO^T leave a lane holding ONE query
//                    column; dQ^T += K^T dS^T with K^T from the LDS transpose read.
// The score recomputation is done in both kernels (7 contractions for 5 counted ones).
#include "a2d_mfma.hpp"

namespace a2d {
namespace {

using namespace mfma;

constexpr int kThreads = 256;
constexpr int BK = 128;   // keys per workgroup (dkdv) / queries per workgroup (dq)
constexpr int BS = 64;    // rows of the streamed operand per step

// stores a transposed accumulator (lane = one output row, registers = 4-column groups)
__device__ __forceinline__ void store_acc_t(float* __restrict__ out_row, const f32x16 (&acc)[4],
                                            int half, float mul) {
#pragma unroll
  for (int ht = 0; ht < 4; ++ht)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4 v = {acc[ht][4 * g] * mul, acc[ht][4 * g + 1] * mul, acc[ht][4 * g + 2] * mul,
                 acc[ht][4 * g + 3] * mul};
      *reinterpret_cast<f32x4*>(out_row + 32 * ht + 8 * g + 4 * half) = v;
    }
}

// ------------------------------------------------------------------ dK, dV
// LDS: [buf]{ Q tile 16 KB, dO tile 16 KB, lse*log2e [64] f32, delta [64] f32 }
constexpr int DKDV_BUF = 2 * TILE64_BYTES + 2 * BS * 4;
constexpr int DKDV_LDS = 2 * DKDV_BUF;

__global__ __launch_bounds__(kThreads, 1) void bwd_dkdv_kernel(
    a2d_tile_desc d, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ delta, float* __restrict__ dK, float* __restrict__ dV) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  int head, blk;
  if (!xcd_map(d.heads, (d.nkv + BK - 1) / BK, head, blk)) return;
  const int k0 = blk * BK;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int half = lane >> 5, l32 = lane & 31;
  Q += (int64_t)head * d.nq * H;
  dO += (int64_t)head * d.nq * H;
  K += (int64_t)head * d.nkv * H;
  V += (int64_t)head * d.nkv * H;
  lse += (int64_t)head * d.nq;
  delta += (int64_t)head * d.nq;
  FragAddr fa;
  fa.init(lane);

  // ---- K^T / V^T B fragments of this wave's 32 keys: lane = key, h = 16 st + 8 half + 0..7
  const int key = k0 + wave * 32 + l32;
  bf16x8 kf[8], vf[8];
  {
    const bool ok = key < d.nkv;
    const int64_t off = (int64_t)(ok ? key : 0) * H + 8 * half;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      u32x4 a = *reinterpret_cast<const u32x4*>(K + off + 16 * st);
      u32x4 b = *reinterpret_cast<const u32x4*>(V + off + 16 * st);
      if (!ok) { a = u32x4{0, 0, 0, 0}; b = u32x4{0, 0, 0, 0}; }
      kf[st] = __builtin_bit_cast(bf16x8, a);
      vf[st] = __builtin_bit_cast(bf16x8, b);
    }
  }
  wait_vmem_all();
  f32x16 dk[4], dv[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) { dk[t] = zero16(); dv[t] = zero16(); }

  // query i sees key r iff i >= r - rel  (local indices), rel = q_off - kv_off
  const int64_t rel = d.q_off - d.kv_off;
  int i_begin = 0;                      // first query row that sees key k0 (the block's first key)
  if (d.causal) {
    const int64_t f = (int64_t)k0 - rel;
    i_begin = f <= 0 ? 0 : (f >= d.nq ? d.nq : (int)f);
  }
  const int i_start = (i_begin / BS) * BS;
  const int nsteps = (d.nq - i_start + BS - 1) / BS;     // 0 if no row sees the block
  const int wk_first = k0 + wave * 32, wk_last = wk_first + 31;
  // first query row seeing this lane's key (rows below it are masked); nq if the key is padding
  int my_first = 0;
  if (d.causal) {
    const int64_t f = (int64_t)key - rel;
    my_first = f <= 0 ? 0 : (f >= d.nq ? d.nq : (int)f);
  }
  if (key >= d.nkv) my_first = d.nq;
  const float c = d.scale * kLog2e;

  Stage64 qst, gst;
  float stat = 0.f;
  auto load_step = [&](int i0) {
    qst.load(Q, i0, d.nq, tid);
    gst.load(dO, i0, d.nq, tid);
    if (tid < BS) {
      const int i = i0 + tid;
      const float v = (i < d.nq) ? lse[i] : INFINITY;
      stat = (v == -INFINITY) ? INFINITY : v * kLog2e;     // +inf makes exp2(s - stat) = 0
    } else if (tid < 2 * BS) {
      const int i = i0 + tid - BS;
      stat = (i < d.nq) ? delta[i] : 0.f;
    }
  };
  auto store_step = [&](char* buf) {
    qst.store(buf, tid);
    gst.store(buf + TILE64_BYTES, tid);
    if (tid < 2 * BS) reinterpret_cast<float*>(buf + 2 * TILE64_BYTES)[tid] = stat;
  };

  if (nsteps > 0) {
    load_step(i_start);
    store_step(lds);
  }
  __syncthreads();

  for (int j = 0; j < nsteps; ++j) {
    const int i0 = i_start + j * BS;
    const char* qs = lds + (j & 1) * DKDV_BUF;
    const char* gs = qs + TILE64_BYTES;
    const float* lse_s = reinterpret_cast<const float*>(qs + 2 * TILE64_BYTES);
    const float* del_s = lse_s + BS;
    if (j + 1 < nsteps) load_step(i0 + BS);

#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int qs0 = i0 + 32 * sub;                          // first query row of the sub-block
      // skip when no (query, key) pair of this 32 x 32 piece is visible
      const bool any_vis = !d.causal || ((int64_t)qs0 + 31 + rel >= wk_first);
      if (qs0 < d.nq && any_vis) {
        f32x16 s = zero16(), dp = zero16();
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          s = mma(read_nat(qs, fa, 32 * sub, st), kf[st], s);
          dp = mma(read_nat(gs, fa, 32 * sub, st), vf[st], dp);
        }
        // register r <-> query qs0 + 8*(r>>2) + 4*half + (r&3); lane <-> key
        const bool need_mask = (wk_last >= d.nkv) || (d.causal && ((int64_t)qs0 + rel < wk_last));
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + 32 * sub + 8 * g + 4 * half);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(del_s + 32 * sub + 8 * g + 4 * half);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * g + e;
            float p = fast_exp2(fmaf(s[r], c, -l4[e]));
            if (need_mask && (qs0 + 8 * g + 4 * half + e < my_first)) p = 0.f;
            s[r] = p;
            dp[r] = p * (dp[r] - d4[e]);
          }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 pb = pack8(s, 8 * u);
          const bf16x8 dsb = pack8(dp, 8 * u);
#pragma unroll
          for (int ht = 0; ht < 4; ++ht) {
            dv[ht] = mma(read_tr(gs, fa, 32 * sub + 16 * u, ht), pb, dv[ht]);
            dk[ht] = mma(read_tr(qs, fa, 32 * sub + 16 * u, ht), dsb, dk[ht]);
          }
        }
      }
    }
    if (j + 1 < nsteps) store_step(lds + ((j + 1) & 1) * DKDV_BUF);
    __syncthreads();
  }

  if (key < d.nkv) {
    const int64_t row = (int64_t)head * d.nkv + key;
    store_acc_t(dK + row * H, dk, half, d.scale);
    store_acc_t(dV + row * H, dv, half, 1.0f);
  }
}

// ---------------------------------------------------------------------- dQ
// LDS: [buf]{ K tile 16 KB, V tile 16 KB }
constexpr int DQ_LDS = 4 * TILE64_BYTES;

__global__ __launch_bounds__(kThreads, 2) void bwd_dq_kernel(
    a2d_tile_desc d, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ delta, float* __restrict__ dQ) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int nqb = (d.nq + BK - 1) / BK;
  int head, blk;
  if (!xcd_map(d.heads, nqb, head, blk)) return;
  const int q0 = (nqb - 1 - blk) * BK;            // heavy blocks first under a causal mask
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int half = lane >> 5, l32 = lane & 31;
  Q += (int64_t)head * d.nq * H;
  dO += (int64_t)head * d.nq * H;
  K += (int64_t)head * d.nkv * H;
  V += (int64_t)head * d.nkv * H;
  FragAddr fa;
  fa.init(lane);

  const int q_row = q0 + wave * 32 + l32;
  const bool q_ok = q_row < d.nq;
  bf16x8 qf[8], gf[8];
  {
    const int64_t off = (int64_t)(q_ok ? q_row : 0) * H + 8 * half;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      u32x4 a = *reinterpret_cast<const u32x4*>(Q + off + 16 * st);
      u32x4 b = *reinterpret_cast<const u32x4*>(dO + off + 16 * st);
      if (!q_ok) { a = u32x4{0, 0, 0, 0}; b = u32x4{0, 0, 0, 0}; }
      qf[st] = __builtin_bit_cast(bf16x8, a);
      gf[st] = __builtin_bit_cast(bf16x8, b);
    }
  }
  float lse2 = INFINITY, del = 0.f;            // +inf: exp2(s - lse2) = 0 for padding / empty rows
  if (q_ok) {
    const float v = lse[(int64_t)head * d.nq + q_row];
    lse2 = (v == -INFINITY) ? INFINITY : v * kLog2e;
    del = delta[(int64_t)head * d.nq + q_row];
  }
  wait_vmem_all();

  const int64_t rel = d.q_off - d.kv_off;
  auto vis_count = [&](int i) -> int {
    if (!d.causal) return d.nkv;
    const int64_t v = (int64_t)i + rel + 1;
    return v <= 0 ? 0 : (v < d.nkv ? (int)v : d.nkv);
  };
  const int blk_last = min(q0 + BK, d.nq) - 1;
  const int nblk = (vis_count(blk_last) + BS - 1) / BS;
  const int w_first = q0 + wave * 32;
  const int w_last = min(w_first + 31, d.nq - 1);
  const int nvis_wave = (w_first < d.nq) ? vis_count(w_last) : 0;
  const int nfull_wave = (w_first < d.nq) ? vis_count(w_first) : 0;
  const int my_vis = q_ok ? vis_count(q_row) : 0;
  const float c = d.scale * kLog2e;

  f32x16 dq[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) dq[t] = zero16();

  Stage64 kst, vst;
  if (nblk > 0) {
    kst.load(K, 0, d.nkv, tid);
    vst.load(V, 0, d.nkv, tid);
    kst.store(lds, tid);
    vst.store(lds + TILE64_BYTES, tid);
  }
  __syncthreads();

  for (int j = 0; j < nblk; ++j) {
    const int k0 = j * BS;
    const char* ks = lds + (j & 1) * 2 * TILE64_BYTES;
    const char* vs = ks + TILE64_BYTES;
    if (j + 1 < nblk) {
      kst.load(K, k0 + BS, d.nkv, tid);
      vst.load(V, k0 + BS, d.nkv, tid);
    }
    if (k0 < nvis_wave) {
      const bool need_mask = k0 + BS > nfull_wave;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x16 s = zero16(), dp = zero16();
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          s = mma(read_nat(ks, fa, 32 * t, st), qf[st], s);
          dp = mma(read_nat(vs, fa, 32 * t, st), gf[st], dp);
        }
        // register r <-> key k0 + 32 t + 8*(r>>2) + 4*half + (r&3); lane <-> query
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = fast_exp2(fmaf(s[r], c, -lse2));
          if (need_mask && (k0 + 32 * t + 8 * (r >> 2) + 4 * half + (r & 3) >= my_vis)) p = 0.f;
          dp[r] = p * (dp[r] - del);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 dsb = pack8(dp, 8 * u);
#pragma unroll
          for (int ht = 0; ht < 4; ++ht) dq[ht] = mma(read_tr(ks, fa, 32 * t + 16 * u, ht), dsb, dq[ht]);
        }
      }
    }
    if (j + 1 < nblk) {
      char* nk = lds + ((j + 1) & 1) * 2 * TILE64_BYTES;
      kst.store(nk, tid);
      vst.store(nk + TILE64_BYTES, tid);
    }
    __syncthreads();
  }
  if (q_ok) store_acc_t(dQ + ((int64_t)head * d.nq + q_row) * H, dq, half, d.scale);
}

}  // namespace

bool bwd_mfma_supported(const a2d_tile_desc& d) {
  return d.dtype == A2D_BF16 && d.hdim == mfma::H;
}

hipError_t launch_bwd_mfma(const a2d_tile_desc& d, const void* Q, const void* K, const void* V,
                           const void* dO, const float* lse, const float* delta, float* dQ,
                           float* dK, float* dV, hipStream_t s) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dkdv_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, DKDV_LDS);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dq_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, DQ_LDS);
  if (e != hipSuccess) return e;
  dim3 block(kThreads);
  dim3 grid_kv(xcd_grid(d.heads, (d.nkv + BK - 1) / BK)), grid_q(xcd_grid(d.heads, (d.nq + BK - 1) / BK));
  hipLaunchKernelGGL(bwd_dkdv_kernel, grid_kv, block, DKDV_LDS, s, d, (const bf16_t*)Q,
                     (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dK, dV);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dq_kernel, grid_q, block, DQ_LDS, s, d, (const bf16_t*)Q, (const bf16_t*)K,
                     (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dQ);
  return hipGetLastError();
}

}  // namespace a2d
