// Generic tile kernels: fp32 arithmetic on the vector ALUs, for fp32 or bf16
// inputs, any nq / nkv, H in {64, 80, 96, 128}.  They serve the fp32 path and every shape
// the MFMA kernels do not cover.  Structure: a 16 x 16 thread grid computes
// register-blocked score tiles out of LDS-resident operand tiles (all widened to
// fp32, rows padded by one word against bank conflicts); probabilities go through
// LDS to the second contraction.
//
// Forward  : Sec. 3.1, Eq. (3), evaluated block by block with the recurrence of
//            Sec. 2.2.
// Backward : the per-tile gradient call of Alg. 3 line 3 with P = exp(S - lse),
//            split into a kernel that owns key rows (dK, dV) and one that owns
//            query rows (dQ), so that no output needs atomics.
#include "a2d_common.hpp"

namespace a2d {
namespace {

constexpr int kThreads = 256;

// dst[r][h] (row stride ld floats) = src row (row0 + r) widened to fp32, zero for rows >= nrows
// (src rows are `stride` elements apart)
template <typename T, int H>
__device__ __forceinline__ void load_tile(float* dst, int ld, const T* __restrict__ src, int64_t stride,
                                          int row0, int nrows, int tile_rows) {
  for (int idx = threadIdx.x; idx < tile_rows * H; idx += kThreads) {
    const int r = idx / H, h = idx - r * H;
    const int g = row0 + r;
    dst[r * ld + h] = (g < nrows) ? to_f32(src[(int64_t)g * stride + h]) : 0.f;
  }
}

__device__ __forceinline__ float group16_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 1, 64));
  v = fmaxf(v, __shfl_xor(v, 2, 64));
  v = fmaxf(v, __shfl_xor(v, 4, 64));
  v = fmaxf(v, __shfl_xor(v, 8, 64));
  return v;
}
__device__ __forceinline__ float group16_sum(float v) {
  v += __shfl_xor(v, 1, 64);
  v += __shfl_xor(v, 2, 64);
  v += __shfl_xor(v, 4, 64);
  v += __shfl_xor(v, 8, 64);
  return v;
}

// number of leading keys of the tile that at least one of the query rows
// [.., q_last] can see under the causal mask (all nkv without a mask)
// (with several sub-blocks: one past the last key that any of them shows to row q_last)
__device__ __forceinline__ int visible_keys(const a2d_tile_desc& d, const SegList& g, int q_last) {
  if (!d.causal) return d.nkv;
  int nvis = 0;
  for (int s = 0; s < g.n; ++s) {
    const int64_t v = (int64_t)q_last + g.rel[s] + 1;          // visible keys of sub-block s
    const int vs = v <= 0 ? 0 : (v < g.rows[s] ? (int)v : g.rows[s]);
    if (vs > 0) nvis = g.start[s] + vs;
  }
  return nvis;
}

// ------------------------------------------------------------------ forward
template <typename T, int H>
__global__ __launch_bounds__(kThreads) void fwd_generic_kernel(
    a2d_tile_desc d, SegList g, const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    float* __restrict__ O_part, float* __restrict__ m_out, float* __restrict__ l_out) {
  constexpr int BM = 64, BN = 64, LD = H + 1, HB = H / 16;
  extern __shared__ float smem[];
  float* Qs = smem;                 // [BM][LD]
  float* Ks = Qs + BM * LD;         // [BN][LD]
  float* Vs = Ks + BN * LD;         // [BN][H]
  float* Ps = Vs + BN * H;          // [BM][BN + 1]
  const int head = blockIdx.y;
  const int q0 = blockIdx.x * BM;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
  Q += (int64_t)head * d.lq.head;
  K += (int64_t)(head / g.group) * d.lk.head;
  V += (int64_t)(head / g.group) * d.lv.head;

  load_tile<T, H>(Qs, LD, Q, d.lq.row, q0, d.nq, BM);

  float o[4][HB];
  float mi[4], li[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    mi[a] = -INFINITY; li[a] = 0.f;
#pragma unroll
    for (int b = 0; b < HB; ++b) o[a][b] = 0.f;
    const int gi = q0 + ty * 4 + a;
    if (g.acc && gi < d.nq) {          // continue from the triple already in the output buffers
      const int64_t row = (int64_t)head * d.nq + gi;
      mi[a] = m_out[row];
      li[a] = (tx == 0) ? l_out[row] : 0.f;     // the lanes' shares are summed at the end
#pragma unroll
      for (int b = 0; b < HB; ++b) o[a][b] = O_part[row * H + tx + 16 * b];
    }
  }
  const int q_last = min(q0 + BM, d.nq) - 1;
  const int nvis = visible_keys(d, g, q_last);

  for (int k0 = 0; k0 < nvis; k0 += BN) {
    __syncthreads();
    load_tile<T, H>(Ks, LD, K, d.lk.row, k0, d.nkv, BN);
    load_tile<T, H>(Vs, H, V, d.lv.row, k0, d.nkv, BN);
    __syncthreads();
    float s[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) s[a][b] = 0.f;
    for (int h = 0; h < H; ++h) {
      float qv[4], kv[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) qv[a] = Qs[(ty * 4 + a) * LD + h];
#pragma unroll
      for (int b = 0; b < 4; ++b) kv[b] = Ks[(tx + 16 * b) * LD + h];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) s[a][b] = fmaf(qv[a], kv[b], s[a][b]);
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int gi = q0 + ty * 4 + a;
      float rmax = -INFINITY;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int c = k0 + tx + 16 * b;
        const bool vis = (c < d.nkv) && (!d.causal || seg_visible(g, gi, c));
        s[a][b] = vis ? s[a][b] * d.scale : -INFINITY;
        rmax = fmaxf(rmax, s[a][b]);
      }
      rmax = group16_max(rmax);
      const float m_new = fmaxf(mi[a], rmax);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = fast_exp2((mi[a] - m_use) * kLog2e);
      float rsum = 0.f;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const float p = fast_exp2((s[a][b] - m_use) * kLog2e);
        rsum += p;
        Ps[(ty * 4 + a) * (BN + 1) + tx + 16 * b] = p;
      }
      li[a] = li[a] * alpha + rsum;   // this lane's share; lanes are summed at the end
      mi[a] = m_new;
#pragma unroll
      for (int b = 0; b < HB; ++b) o[a][b] *= alpha;
    }
    __syncthreads();
    for (int c = 0; c < BN; ++c) {
      float pv[4], vv[HB];
#pragma unroll
      for (int a = 0; a < 4; ++a) pv[a] = Ps[(ty * 4 + a) * (BN + 1) + c];
#pragma unroll
      for (int b = 0; b < HB; ++b) vv[b] = Vs[c * H + tx + 16 * b];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < HB; ++b) o[a][b] = fmaf(pv[a], vv[b], o[a][b]);
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int gi = q0 + ty * 4 + a;
    const float lsum = group16_sum(li[a]);
    if (gi < d.nq && g.norm) {
      // normalised partial in the input dtype and lse' = m + ln l
      const int64_t row = (int64_t)head * d.nq + gi;
      const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
      T* on = reinterpret_cast<T*>(O_part);
#pragma unroll
      for (int b = 0; b < HB; ++b) on[row * H + tx + 16 * b] = (T)(o[a][b] * inv);
      if (tx == 0) m_out[row] = lsum > 0.f ? mi[a] + logf(lsum) : -INFINITY;
    } else if (gi < d.nq) {
      const int64_t row = (int64_t)head * d.nq + gi;
#pragma unroll
      for (int b = 0; b < HB; ++b) O_part[row * H + tx + 16 * b] = o[a][b];
      if (tx == 0) { m_out[row] = mi[a]; l_out[row] = lsum; }
    }
  }
}

// ------------------------------------------------------------- backward: dK, dV
template <typename T, int H>
__global__ __launch_bounds__(kThreads) void bwd_dkdv_generic_kernel(
    a2d_tile_desc d, SegList g, const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ delta,
    float* __restrict__ dK, float* __restrict__ dV) {
  constexpr int BK = 64, BQ = 32, LD = H + 1, HB = H / 16, LP = BK + 1;
  extern __shared__ float smem[];
  float* Ks = smem;                // [BK][LD]
  float* Vs = Ks + BK * LD;        // [BK][LD]
  float* Qs = Vs + BK * LD;        // [BQ][LD]
  float* dOs = Qs + BQ * LD;       // [BQ][LD]
  float* Ps = dOs + BQ * LD;       // [BQ][LP]
  float* dSs = Ps + BQ * LP;       // [BQ][LP]
  const int head = blockIdx.y;     // key/value head: its g.group query heads follow one another in Q, dO, lse, delta
  const int k0 = blockIdx.x * BK;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
  Q += (int64_t)head * g.group * d.lq.head;
  dO += (int64_t)head * g.group * d.ldo.head;
  K += (int64_t)head * d.lk.head;
  V += (int64_t)head * d.lv.head;
  lse += (int64_t)head * g.group * d.nq;
  delta += (int64_t)head * g.group * d.nq;

  load_tile<T, H>(Ks, LD, K, d.lk.row, k0, d.nkv, BK);
  load_tile<T, H>(Vs, LD, V, d.lv.row, k0, d.nkv, BK);

  float dk[4][HB], dv[4][HB];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < HB; ++b) { dk[a][b] = 0.f; dv[a][b] = 0.f; }

  // first query row that can see key k0 (rows before it see none of this block's keys)
  // (with several sub-blocks: the earliest such row over the sub-blocks this key block touches)
  int i_first = 0;
  if (d.causal) {
    i_first = d.nq;
    const int k_end = min(k0 + BK, d.nkv);
    for (int sb = 0; sb < g.n; ++sb) {
      const int a = max(k0, g.start[sb]), b = min(k_end, g.start[sb] + g.rows[sb]);
      if (a >= b) continue;
      const int64_t f = (int64_t)(a - g.start[sb]) - g.rel[sb];      // first row that sees key a
      const int fr = f <= 0 ? 0 : (f >= d.nq ? d.nq : (int)f);
      i_first = min(i_first, fr);
    }
  }
  for (int qh = 0; qh < g.group; ++qh, Q += d.lq.head, dO += d.ldo.head, lse += d.nq, delta += d.nq)
  for (int i0 = (i_first / BQ) * BQ; i0 < d.nq; i0 += BQ) {
    __syncthreads();
    load_tile<T, H>(Qs, LD, Q, d.lq.row, i0, d.nq, BQ);
    load_tile<T, H>(dOs, LD, dO, d.ldo.row, i0, d.nq, BQ);
    __syncthreads();
    float s[2][4], dp[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) { s[a][b] = 0.f; dp[a][b] = 0.f; }
    for (int h = 0; h < H; ++h) {
      float qv[2], gv[2], kv[4], vv[4];
#pragma unroll
      for (int a = 0; a < 2; ++a) { qv[a] = Qs[(ty * 2 + a) * LD + h]; gv[a] = dOs[(ty * 2 + a) * LD + h]; }
#pragma unroll
      for (int b = 0; b < 4; ++b) { kv[b] = Ks[(tx + 16 * b) * LD + h]; vv[b] = Vs[(tx + 16 * b) * LD + h]; }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          s[a][b] = fmaf(qv[a], kv[b], s[a][b]);
          dp[a][b] = fmaf(gv[a], vv[b], dp[a][b]);
        }
    }
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      const int i = i0 + ty * 2 + a;
      const bool row_ok = i < d.nq;
      const float lse_i = row_ok ? lse[i] : -INFINITY;
      const float del_i = row_ok ? delta[i] : 0.f;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int c = k0 + tx + 16 * b;
        const bool vis = row_ok && (lse_i != -INFINITY) && (c < d.nkv) &&
                         (!d.causal || seg_visible(g, i, c));
        const float p = vis ? fast_exp2((s[a][b] * d.scale - lse_i) * kLog2e) : 0.f;
        Ps[(ty * 2 + a) * LP + tx + 16 * b] = p;
        dSs[(ty * 2 + a) * LP + tx + 16 * b] = p * (dp[a][b] - del_i);
      }
    }
    __syncthreads();
    for (int i = 0; i < BQ; ++i) {
      float pv[4], dsv[4], gv[HB], qv[HB];
#pragma unroll
      for (int a = 0; a < 4; ++a) { pv[a] = Ps[i * LP + ty * 4 + a]; dsv[a] = dSs[i * LP + ty * 4 + a]; }
#pragma unroll
      for (int b = 0; b < HB; ++b) { gv[b] = dOs[i * LD + tx + 16 * b]; qv[b] = Qs[i * LD + tx + 16 * b]; }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < HB; ++b) {
          dv[a][b] = fmaf(pv[a], gv[b], dv[a][b]);
          dk[a][b] = fmaf(dsv[a], qv[b], dk[a][b]);
        }
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int c = k0 + ty * 4 + a;
    if (c < d.nkv) {
      const int64_t row = (int64_t)head * d.nkv + c;
#pragma unroll
      for (int b = 0; b < HB; ++b) {
        dK[row * H + tx + 16 * b] = dk[a][b] * d.scale;
        dV[row * H + tx + 16 * b] = dv[a][b];
      }
    }
  }
}

// ---------------------------------------------------------------- backward: dQ
template <typename T, int H>
__global__ __launch_bounds__(kThreads) void bwd_dq_generic_kernel(
    a2d_tile_desc d, SegList g, const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ delta,
    float* __restrict__ dQ) {
  constexpr int BQ = 64, BK = 32, LD = H + 1, HB = H / 16, LP = BK + 1;
  extern __shared__ float smem[];
  float* Qs = smem;               // [BQ][LD]
  float* dOs = Qs + BQ * LD;      // [BQ][LD]
  float* Ks = dOs + BQ * LD;      // [BK][LD]
  float* Vs = Ks + BK * LD;       // [BK][LD]
  float* dSs = Vs + BK * LD;      // [BQ][LP]
  const int head = blockIdx.y;
  const int q0 = blockIdx.x * BQ;
  const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
  Q += (int64_t)head * d.lq.head;
  dO += (int64_t)head * d.ldo.head;
  K += (int64_t)(head / g.group) * d.lk.head;
  V += (int64_t)(head / g.group) * d.lv.head;
  lse += (int64_t)head * d.nq;
  delta += (int64_t)head * d.nq;

  load_tile<T, H>(Qs, LD, Q, d.lq.row, q0, d.nq, BQ);
  load_tile<T, H>(dOs, LD, dO, d.ldo.row, q0, d.nq, BQ);

  float dq[4][HB];
  float lse_i[4], del_i[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int i = q0 + ty * 4 + a;
    lse_i[a] = (i < d.nq) ? lse[i] : -INFINITY;
    del_i[a] = (i < d.nq) ? delta[i] : 0.f;
#pragma unroll
    for (int b = 0; b < HB; ++b) dq[a][b] = 0.f;
  }
  const int q_last = min(q0 + BQ, d.nq) - 1;
  const int nvis = visible_keys(d, g, q_last);

  for (int k0 = 0; k0 < nvis; k0 += BK) {
    __syncthreads();
    load_tile<T, H>(Ks, LD, K, d.lk.row, k0, d.nkv, BK);
    load_tile<T, H>(Vs, LD, V, d.lv.row, k0, d.nkv, BK);
    __syncthreads();
    float s[4][2], dp[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) { s[a][b] = 0.f; dp[a][b] = 0.f; }
    for (int h = 0; h < H; ++h) {
      float qv[4], gv[4], kv[2], vv[2];
#pragma unroll
      for (int a = 0; a < 4; ++a) { qv[a] = Qs[(ty * 4 + a) * LD + h]; gv[a] = dOs[(ty * 4 + a) * LD + h]; }
#pragma unroll
      for (int b = 0; b < 2; ++b) { kv[b] = Ks[(tx + 16 * b) * LD + h]; vv[b] = Vs[(tx + 16 * b) * LD + h]; }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          s[a][b] = fmaf(qv[a], kv[b], s[a][b]);
          dp[a][b] = fmaf(gv[a], vv[b], dp[a][b]);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int gi = q0 + ty * 4 + a;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int c = k0 + tx + 16 * b;
        const bool vis = (lse_i[a] != -INFINITY) && (c < d.nkv) && (!d.causal || seg_visible(g, gi, c));
        const float p = vis ? fast_exp2((s[a][b] * d.scale - lse_i[a]) * kLog2e) : 0.f;
        dSs[(ty * 4 + a) * LP + tx + 16 * b] = p * (dp[a][b] - del_i[a]);
      }
    }
    __syncthreads();
    for (int c = 0; c < BK; ++c) {
      float dsv[4], kv[HB];
#pragma unroll
      for (int a = 0; a < 4; ++a) dsv[a] = dSs[(ty * 4 + a) * LP + c];
#pragma unroll
      for (int b = 0; b < HB; ++b) kv[b] = Ks[c * LD + tx + 16 * b];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < HB; ++b) dq[a][b] = fmaf(dsv[a], kv[b], dq[a][b]);
    }
  }
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int i = q0 + ty * 4 + a;
    if (i < d.nq) {
      const int64_t row = (int64_t)head * d.nq + i;
#pragma unroll
      for (int b = 0; b < HB; ++b) {
        const float v = dq[a][b] * d.scale;
        dQ[row * H + tx + 16 * b] = g.acc ? dQ[row * H + tx + 16 * b] + v : v;
      }
    }
  }
}

// --------------------------------------------------- delta = rowsum(dO o O)
// LPR lanes share a row, each reading 16 bytes of O and of dO per step.
// (O and dO are [heads][nq][H] tensors with the strides lo / ldo; delta is plain [heads][nq])
template <typename T>
__global__ __launch_bounds__(kThreads) void delta_kernel(int64_t rows, int nq, int H, int lpr, a2d_layout lo,
                                                         a2d_layout ldo, const T* __restrict__ O,
                                                         const T* __restrict__ dO,
                                                         float* __restrict__ delta) {
  constexpr int EPL = 16 / sizeof(T);          // elements per lane per load
  // lpr lanes per row: the power of two that covers H / EPL loads (8 .. 32); for head sizes that
  // are not powers of two the surplus lanes of a row idle
  const int nload = H / EPL;
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t row = idx / lpr;
  const int c = (int)(idx - row * lpr);
  float acc = 0.f;
  if (row < rows && c < nload) {
    const int64_t head = row / nq, r = row - head * nq;
    const T* o = O + head * lo.head + r * lo.row + c * EPL;
    const T* g = dO + head * ldo.head + r * ldo.row + c * EPL;
    const u32x4 ow = *reinterpret_cast<const u32x4*>(o);
    const u32x4 gw = *reinterpret_cast<const u32x4*>(g);
    const T* ov = reinterpret_cast<const T*>(&ow);
    const T* gv = reinterpret_cast<const T*>(&gw);
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc = fmaf(to_f32(ov[e]), to_f32(gv[e]), acc);
  }
  for (int o = 1; o < lpr; o <<= 1) acc += __shfl_xor(acc, o, 64);
  if (row < rows && c == 0) delta[row] = acc;
}

template <typename K>
hipError_t set_lds(K kernel, size_t bytes) {
  return ensure_dynamic_lds(reinterpret_cast<const void*>(kernel), (int)bytes);
}

template <typename T, int H>
hipError_t fwd_launch(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K, const void* V,
                      float* O_part, float* m, float* l, hipStream_t s) {
  constexpr size_t lds = sizeof(float) * (64 * (H + 1) * 2 + 64 * H + 64 * 65);
  if (ph == PREPARE) return set_lds(fwd_generic_kernel<T, H>, lds);
  dim3 grid((d.nq + 63) / 64, d.heads), block(kThreads);
  A2D_LAUNCH((fwd_generic_kernel<T, H>), grid, block, lds, s, d, g, (const T*)Q, (const T*)K,
                     (const T*)V, O_part, m, l);
  return hipGetLastError();
}

template <typename T, int H>
hipError_t bwd_launch(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K, const void* V,
                      const void* dO, const float* lse, const float* delta, float* dQ, float* dK,
                      float* dV, hipStream_t s) {
  constexpr size_t lds_kv = sizeof(float) * (2 * 64 * (H + 1) + 2 * 32 * (H + 1) + 2 * 32 * 65);
  constexpr size_t lds_q = sizeof(float) * (2 * 64 * (H + 1) + 2 * 32 * (H + 1) + 64 * 33);
  if (ph == PREPARE) {
    const hipError_t e = set_lds(bwd_dkdv_generic_kernel<T, H>, lds_kv);
    return e != hipSuccess ? e : set_lds(bwd_dq_generic_kernel<T, H>, lds_q);
  }
  dim3 block(kThreads);
  dim3 grid_kv((d.nkv + 63) / 64, d.heads / g.group), grid_q((d.nq + 63) / 64, d.heads);
  A2D_LAUNCH((bwd_dkdv_generic_kernel<T, H>), grid_kv, block, lds_kv, s, d, g, (const T*)Q,
                     (const T*)K, (const T*)V, (const T*)dO, lse, delta, dK, dV);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  A2D_LAUNCH((bwd_dq_generic_kernel<T, H>), grid_q, block, lds_q, s, d, g, (const T*)Q,
                     (const T*)K, (const T*)V, (const T*)dO, lse, delta, dQ);
  return hipGetLastError();
}

}  // namespace

// head sizes of the paper's models (Table 3): 128, 96, 80; and 64
#define A2D_DISPATCH_H(FN, T, ...)                  \
  switch (d.hdim) {                                 \
    case 128: return FN<T, 128>(__VA_ARGS__);       \
    case 96: return FN<T, 96>(__VA_ARGS__);         \
    case 80: return FN<T, 80>(__VA_ARGS__);         \
    default: return FN<T, 64>(__VA_ARGS__);         \
  }

hipError_t launch_fwd_generic(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                              const void* V, float* O_part, float* m, float* l, hipStream_t s) {
  if (d.dtype == A2D_BF16) { A2D_DISPATCH_H(fwd_launch, bf16_t, ph, d, g, Q, K, V, O_part, m, l, s) }
  A2D_DISPATCH_H(fwd_launch, float, ph, d, g, Q, K, V, O_part, m, l, s)
}

hipError_t launch_bwd_generic(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                              const void* V, const void* dO, const float* lse, const float* delta, float* dQ,
                              float* dK, float* dV, hipStream_t s) {
  if (d.dtype == A2D_BF16) { A2D_DISPATCH_H(bwd_launch, bf16_t, ph, d, g, Q, K, V, dO, lse, delta, dQ, dK, dV, s) }
  A2D_DISPATCH_H(bwd_launch, float, ph, d, g, Q, K, V, dO, lse, delta, dQ, dK, dV, s)
}
#undef A2D_DISPATCH_H

hipError_t launch_delta(const a2d_tile_desc& d, const void* O, const void* dO, float* delta, hipStream_t s) {
  const int dtype = d.dtype, hdim = d.hdim;
  const int64_t rows = (int64_t)d.heads * d.nq;
  const int epl = dtype == A2D_BF16 ? 8 : 4;
  int lpr = 1;
  while (lpr < hdim / epl) lpr <<= 1;
  const int64_t threads = rows * lpr;
  dim3 grid((unsigned)((threads + kThreads - 1) / kThreads)), block(kThreads);
  if (dtype == A2D_BF16)
    A2D_LAUNCH((delta_kernel<bf16_t>), grid, block, 0, s, rows, d.nq, hdim, lpr, d.lo, d.ldo,
                       (const bf16_t*)O, (const bf16_t*)dO, delta);
  else
    A2D_LAUNCH((delta_kernel<float>), grid, block, 0, s, rows, d.nq, hdim, lpr, d.lo, d.ldo,
                       (const float*)O, (const float*)dO, delta);
  return hipGetLastError();
}

}  // namespace a2d
