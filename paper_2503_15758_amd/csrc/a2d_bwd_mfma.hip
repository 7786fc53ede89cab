// bf16 MFMA backward tile kernels for H = 128: the per-tile gradient call of Alg. 3
// line 3 with P = exp(S - lse) rebuilt from the FINAL log-sum-exp of the query block,
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Two kernels, so that every output has exactly one writer and no atomics are needed
// (bitwise reproducible results):
//   bwd_dkdv_kernel  owns key rows.  Workgroup = 4 wavefronts = 128 keys (32 per
//                    wavefront, K and V fragments resident in registers); walks
//                    the query blocks, 64 rows per step, staged through LDS together with
//                    dO, lse and delta.  S = Q K^T and dP = dO V^T leave a lane holding
//                    ONE key column, so P and dS feed dV^T += dO^T P and dK^T += Q^T dS
//                    directly as B operands; dO^T / Q^T come from the LDS transpose read.
//   bwd_dq_kernel    owns query rows.  Workgroup = 4 wavefronts = 128 queries (32 per
//                    wavefront, Q and dO fragments in registers), two workgroups per
//                    compute unit; walks the key blocks, 64 keys per step.  S^T = K Q^T
//                    and dP^T = V dO^T leave a lane holding ONE query column;
//                    dQ^T += K^T dS^T with K^T from the LDS transpose read.
// The dK/dV kernel needs more than 256 VGPRs (128 of accumulators alone) and runs one
// wavefront per SIMD; the dQ kernel keeps two, so one's MFMAs overlap the other's
// exponentials (a single wavefront cannot overlap the two).  In the dK/dV kernel the tiles
// read both ways live in the "dual" LDS layout of a2d_mfma.hpp (every fragment address is a
// per-lane base plus an immediate); the dQ kernel uses the XOR-swizzled layout.  The score recomputation is done in both kernels (7 contractions
// for 5 counted ones).
#include "a2d_mfma.hpp"

namespace a2d {
namespace {

using namespace mfma;

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

__device__ __forceinline__ f32x4 lds_load_f32x4(unsigned addr) {
  return *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>((uintptr_t)addr);
}

// natural fragment x of a dual tile (rows RB .. RB+31 relative to the per-lane bases in `a`)
template <int X>
__device__ __forceinline__ bf16x8 dual_nat(const DualAddr& a, int extra) {
  return lds_load_b128(((X & 1) ? a.nat_o : a.nat_e) + 64 * (X >> 1) + extra);
}

// ------------------------------------------------------------------ dK, dV
constexpr int DK_THREADS = 256;
constexpr int DK_KEYS = 128;      // keys per workgroup
constexpr int BQ = 64;            // query rows per step
// LDS: [buf]{ Q tile, dO tile } (dual layout) | [buf]{ lse*log2e [64], delta [64] }
constexpr int DK_BUF = 2 * DUAL64_BYTES;
constexpr int DK_STAT = 2 * DK_BUF;
constexpr int DK_LDS = DK_STAT + 2 * 2 * BQ * 4;

struct DkCtx {
  f32x16 dk[4], dv[4];
  bf16x8 kf[8], vf[8];  // K^T / V^T fragments of this wavefront's 32 keys
  DualAddr qa;          // Q tile of the current buffer; the dO tile is DUAL64_BYTES further
  unsigned stat;        // lse / delta rows of the current buffer, offset by 16 * half
  float c;
  int my_first;         // first local query row that sees this lane's key
  int half;
};

// One 32-query x 32-key piece; SUB selects the half of the 64-row step.
// A single wavefront per SIMD runs this kernel, so nothing hides LDS latency but the
// instruction order: every fragment is requested about four MFMA pairs before its use
// (rolling prefetch; the LDS wait counter only tracks 15 operations in flight).
template <int SUB, bool MASK>
__device__ __forceinline__ void dkdv_piece(DkCtx& cx, int qs0) {
  constexpr int RB = SUB * 32 * DUAL_LD;
  constexpr int GO = DUAL64_BYTES;            // dO tile behind the Q tile
  bf16x8 qn[4], gn[4];                        // ring of natural fragments, four steps deep
  // (the scheduling fences keep the compiler from sinking the requests back to their uses)
#define A2D_LD1(X)                                                                  \
  qn[(X) & 3] = dual_nat<X>(cx.qa, RB); gn[(X) & 3] = dual_nat<X>(cx.qa, RB + GO); \
  __builtin_amdgcn_sched_barrier(0);
#define A2D_SDP(X) s = mma(qn[(X) & 3], cx.kf[X], s); dp = mma(gn[(X) & 3], cx.vf[X], dp);
  A2D_LD1(0) A2D_LD1(1) A2D_LD1(2) A2D_LD1(3)
  f32x16 s = zero16(), dp = zero16();
  A2D_SDP(0) A2D_LD1(4)
  A2D_SDP(1) A2D_LD1(5)
  A2D_SDP(2) A2D_LD1(6)
  A2D_SDP(3) A2D_LD1(7)
  // transposed fragments of the first 16 query rows: on their way during the exponentials
  bf16x8 gt[4], qt[4];
#define A2D_LD2(HT, U)                                                                                   \
  gt[HT] = lds_load_tr(cx.qa.tr_lo + GO + RB + (U) * 16 * DUAL_LD + 64 * (HT),                            \
                       cx.qa.tr_hi + GO + RB + (U) * 16 * DUAL_LD + 64 * (HT));                           \
  qt[HT] = lds_load_tr(cx.qa.tr_lo + RB + (U) * 16 * DUAL_LD + 64 * (HT),                                 \
                       cx.qa.tr_hi + RB + (U) * 16 * DUAL_LD + 64 * (HT));                                \
  __builtin_amdgcn_sched_barrier(0);
  A2D_SDP(4) A2D_LD2(0, 0)
  A2D_SDP(5) A2D_LD2(1, 0)
  A2D_SDP(6) A2D_LD2(2, 0)
  A2D_SDP(7) A2D_LD2(3, 0)
#undef A2D_SDP
#undef A2D_LD1
  // register r <-> query qs0 + 8*(r>>2) + 4*half + (r&3); lane <-> key
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const f32x4 l4 = lds_load_f32x4(cx.stat + (SUB * 32 + 8 * g) * 4);
    const f32x4 d4 = lds_load_f32x4(cx.stat + (BQ + SUB * 32 + 8 * g) * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int r = 4 * g + e;
      float p = fast_exp2(fmaf(s[r], cx.c, -l4[e]));
      if (MASK && (qs0 + 8 * g + 4 * cx.half + e < cx.my_first)) p = 0.f;
      s[r] = p;
      dp[r] = p * (dp[r] - d4[e]);
    }
  }
  bf16x8 pb[2], dsb[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) { pb[u] = pack8(s, 8 * u); dsb[u] = pack8(dp, 8 * u); }
#define A2D_DVDK(HT, U) cx.dv[HT] = mma(gt[HT], pb[U], cx.dv[HT]); cx.dk[HT] = mma(qt[HT], dsb[U], cx.dk[HT]);
  A2D_DVDK(0, 0) A2D_LD2(0, 1)
  A2D_DVDK(1, 0) A2D_LD2(1, 1)
  A2D_DVDK(2, 0) A2D_LD2(2, 1)
  A2D_DVDK(3, 0) A2D_LD2(3, 1)
  A2D_DVDK(0, 1) A2D_DVDK(1, 1) A2D_DVDK(2, 1) A2D_DVDK(3, 1)
#undef A2D_DVDK
#undef A2D_LD2
}

__global__ __launch_bounds__(DK_THREADS, 1) void bwd_dkdv_kernel(
    a2d_tile_desc d, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ delta, float* __restrict__ dK, float* __restrict__ dV) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
  int head, blk;
  if (!xcd_map(d.heads, (d.nkv + DK_KEYS - 1) / DK_KEYS, head, blk)) return;
  const int k0 = blk * DK_KEYS;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31;
  Q += (int64_t)head * d.nq * H;
  dO += (int64_t)head * d.nq * H;
  K += (int64_t)head * d.nkv * H;
  V += (int64_t)head * d.nkv * H;
  lse += (int64_t)head * d.nq;
  delta += (int64_t)head * d.nq;

  DkCtx cx;
  cx.half = lane >> 5;
  cx.c = d.scale * kLog2e;
  // ---- K^T / V^T B fragments of this wave's 32 keys: lane = key, h = 16 x + 8 half + 0..7.
  // Keys beyond nkv re-read the last key; the mask zeroes their probabilities.
  const int key = k0 + wave * 32 + l32;
  {
    const int64_t off = (int64_t)min(key, d.nkv - 1) * H + 8 * cx.half;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      cx.kf[x] = *reinterpret_cast<const bf16x8*>(K + off + 16 * x);
      cx.vf[x] = *reinterpret_cast<const bf16x8*>(V + off + 16 * x);
    }
  }
  wait_vmem_all();
#pragma unroll
  for (int t = 0; t < 4; ++t) { cx.dk[t] = zero16(); cx.dv[t] = zero16(); }

  // query i sees key r iff i >= r - rel  (local indices), rel = q_off - kv_off
  const int64_t rel = d.q_off - d.kv_off;
  auto first_row = [&](int r) -> int {          // first local query row that sees local key r
    if (!d.causal) return 0;
    const int64_t f = (int64_t)r - rel;
    return f <= 0 ? 0 : (f >= d.nq ? d.nq : (int)f);
  };
  const int i_start = (first_row(k0) / BQ) * BQ;
  const int nsteps = (d.nq - i_start + BQ - 1) / BQ;
  const int wk_first = k0 + wave * 32, wk_last = wk_first + 31;
  cx.my_first = (key < d.nkv) ? first_row(key) : d.nq;       // padding keys see nothing
  const int w_any = first_row(wk_first);                      // rows below see none of the wave's keys
  const int w_all = (wk_last < d.nkv) ? first_row(wk_last) : d.nq;   // rows from here see all of them

  cx.qa.init(lane, lds_base);
  cx.stat = lds_base + DK_STAT + 16 * cx.half;

  // ---- staging of a 64-row step in two halves of 32 rows (16 registers in flight): thread moves
  // chunk (tid & 15) of rows (tid >> 4) + 16 p of a half.  Rows beyond nq re-read the last row;
  // their lse entry is +inf, which makes exp2(s - lse) = 0 (also for rows whose lse is -inf).
  static_assert(DK_THREADS == 256, "staging map assumes 256 threads");
  const int st_row = tid >> 4, st_ch = tid & 15;
  u32x4 qreg[2], greg[2];
  float stat = 0.f;
  bool stat_ok = false;
  auto load_half = [&](int i0, int hf) {
    const gptr_t qb = uniform_gptr(Q + (int64_t)i0 * H);
    const gptr_t gb = uniform_gptr(dO + (int64_t)i0 * H);
    const int last = d.nq - 1 - i0;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const unsigned off = (unsigned)(min(32 * hf + st_row + 16 * p, last) * (H * 2) + st_ch * 16);
      qreg[p] = gload_b128(qb, off);
      greg[p] = gload_b128(gb, off);
    }
    // raw statistic loads only: converting here would make the wave wait for everything just issued
    if (hf == 0 && tid < 2 * BQ) {
      const int i = min(i0 + (tid & (BQ - 1)), d.nq - 1);
      stat = (tid < BQ) ? lse[i] : delta[i];
      stat_ok = (i0 + (tid & (BQ - 1))) < d.nq;
    }
  };
  auto store_half = [&](int buf, int hf) {
    char* b = lds + buf * DK_BUF;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int off = dual_store_off(32 * hf + st_row + 16 * p, st_ch);
      *reinterpret_cast<u32x4*>(b + off) = qreg[p];
      *reinterpret_cast<u32x4*>(b + DUAL64_BYTES + off) = greg[p];
    }
    if (hf == 0 && tid < 2 * BQ) {
      float v = stat;
      if (tid < BQ) v = (!stat_ok || v == -INFINITY) ? INFINITY : v * kLog2e;
      else v = stat_ok ? v : 0.f;
      reinterpret_cast<float*>(lds + DK_STAT + buf * 2 * BQ * 4)[tid] = v;
    }
  };

  if (nsteps > 0) {
    load_half(i_start, 0); store_half(0, 0);
    load_half(i_start, 1); store_half(0, 1);
  }
  __syncthreads();

  for (int j = 0; j < nsteps; ++j) {
    const int i0 = i_start + j * BQ;
    const bool more = j + 1 < nsteps;
    if (more) load_half(i0 + BQ, 0);
    // piece (SUB): rows i0 + 32 SUB .. +31.  Skipped when no row of it sees any key of the wave
    // or it lies beyond nq; masked unless every row sees every key.
    if (i0 + 31 >= w_any && i0 < d.nq) {
      if (i0 >= w_all && i0 + 32 <= d.nq) dkdv_piece<0, false>(cx, i0);
      else dkdv_piece<0, true>(cx, i0);
    }
    if (more) { store_half((j + 1) & 1, 0); load_half(i0 + BQ, 1); }
    if (i0 + 63 >= w_any && i0 + 32 < d.nq) {
      if (i0 + 32 >= w_all && i0 + 64 <= d.nq) dkdv_piece<1, false>(cx, i0 + 32);
      else dkdv_piece<1, true>(cx, i0 + 32);
    }
    if (more) store_half((j + 1) & 1, 1);
    const int tog = (j & 1) ? -DK_BUF : DK_BUF;
    cx.qa.shift(tog);
    cx.stat += (j & 1) ? -2 * BQ * 4 : 2 * BQ * 4;
    __syncthreads();
  }

  if (key < d.nkv) {
    const int64_t row = (int64_t)head * d.nkv + key;
    store_acc_t(dK + row * H, cx.dk, cx.half, d.scale);
    store_acc_t(dV + row * H, cx.dv, cx.half, 1.0f);
  }
}

// ---------------------------------------------------------------------- dQ
constexpr int DQ_THREADS = 256;
constexpr int DQ_ROWS = 128;      // query rows per workgroup
constexpr int BKS = 64;           // keys per step
constexpr int VT_LD = 272;        // V tile row stride (natural reads only)
// LDS: [buf]{ K tile (dual layout), V tile (272-byte rows) }
constexpr int DQ_VT = DUAL64_BYTES;
constexpr int DQ_BUF = DUAL64_BYTES + BKS * VT_LD;
constexpr int DQ_LDS = 2 * DQ_BUF;
constexpr int DQ_RING = 2;        // fragment ring depth (registers are tight: 256 per wavefront)

struct DqCtx {
  f32x16 dq[4];
  bf16x8 qf[8], gf[8];
  DualAddr ka;          // K tile of the current buffer
  unsigned vnat;        // natural-fragment base in the V tile of the current buffer
  float c, lse2, del;
  int my_vis;           // number of leading local keys this lane's query row sees
  int half;
};

// one 32-key x 32-query piece: T selects the half of the 64-key step
template <int T, bool MASK>
__device__ __forceinline__ void dq_piece(DqCtx& cx, int key0) {
  constexpr int RB = T * 32 * DUAL_LD;
  constexpr int VB = T * 32 * VT_LD;
  bf16x8 kr[DQ_RING], vr[DQ_RING];
#define A2D_LD1(X)                                             \
  kr[(X) % DQ_RING] = dual_nat<X>(cx.ka, RB);                  \
  vr[(X) % DQ_RING] = lds_load_b128(cx.vnat + VB + 32 * (X));  \
  __builtin_amdgcn_sched_barrier(0);
#define A2D_SDP(X) s = mma(kr[(X) % DQ_RING], cx.qf[X], s); dp = mma(vr[(X) % DQ_RING], cx.gf[X], dp);
  A2D_LD1(0) A2D_LD1(1)
  f32x16 s = zero16(), dp = zero16();
  A2D_SDP(0) A2D_LD1(2)
  A2D_SDP(1) A2D_LD1(3)
  A2D_SDP(2) A2D_LD1(4)
  A2D_SDP(3) A2D_LD1(5)
  A2D_SDP(4) A2D_LD1(6)
  A2D_SDP(5) A2D_LD1(7)
  // K^T fragments of the first key rows: on their way during the exponentials
  bf16x8 kt[DQ_RING];
#define A2D_LD2(I)                                                                                        \
  kt[(I) % DQ_RING] = lds_load_tr(cx.ka.tr_lo + RB + ((I) >> 2) * 16 * DUAL_LD + 64 * ((I) & 3),          \
                                  cx.ka.tr_hi + RB + ((I) >> 2) * 16 * DUAL_LD + 64 * ((I) & 3));         \
  __builtin_amdgcn_sched_barrier(0);
  A2D_SDP(6) A2D_LD2(0)
  A2D_SDP(7) A2D_LD2(1)
#undef A2D_SDP
#undef A2D_LD1
  // register r <-> key key0 + 8*(r>>2) + 4*half + (r&3); lane <-> query
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float p = fast_exp2(fmaf(s[r], cx.c, -cx.lse2));
    if (MASK && (key0 + 8 * (r >> 2) + 4 * cx.half + (r & 3) >= cx.my_vis)) p = 0.f;
    dp[r] = p * (dp[r] - cx.del);
  }
  bf16x8 dsb[2];
  dsb[0] = pack8(dp, 0);
  dsb[1] = pack8(dp, 8);
  __builtin_amdgcn_sched_barrier(0);
#define A2D_DQ(I) cx.dq[(I) & 3] = mma(kt[(I) % DQ_RING], dsb[(I) >> 2], cx.dq[(I) & 3]);
  A2D_DQ(0) A2D_LD2(2)
  A2D_DQ(1) A2D_LD2(3)
  A2D_DQ(2) A2D_LD2(4)
  A2D_DQ(3) A2D_LD2(5)
  A2D_DQ(4) A2D_LD2(6)
  A2D_DQ(5) A2D_LD2(7)
  A2D_DQ(6) A2D_DQ(7)
#undef A2D_DQ
#undef A2D_LD2
}

__global__ __launch_bounds__(DQ_THREADS, 2) void bwd_dq_kernel(
    a2d_tile_desc d, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ delta, float* __restrict__ dQ) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
  const int nqb = (d.nq + DQ_ROWS - 1) / DQ_ROWS;
  int head, blk;
  if (!xcd_map(d.heads, nqb, head, blk)) return;
  const int q0 = (nqb - 1 - blk) * DQ_ROWS;            // heavy blocks first under a causal mask
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31;
  Q += (int64_t)head * d.nq * H;
  dO += (int64_t)head * d.nq * H;
  K += (int64_t)head * d.nkv * H;
  V += (int64_t)head * d.nkv * H;

  DqCtx cx;
  cx.half = lane >> 5;
  cx.c = d.scale * kLog2e;
  const int q_row = q0 + wave * 32 + l32;
  const bool q_ok = q_row < d.nq;
  const int q_ld = min(q_row, d.nq - 1);         // rows beyond nq re-read the last row, lse2 = +inf
  {
    const int64_t off = (int64_t)q_ld * H + 8 * cx.half;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      cx.qf[x] = *reinterpret_cast<const bf16x8*>(Q + off + 16 * x);
      cx.gf[x] = *reinterpret_cast<const bf16x8*>(dO + off + 16 * x);
    }
    const float v = lse[(int64_t)head * d.nq + q_ld];
    cx.lse2 = (!q_ok || v == -INFINITY) ? INFINITY : v * kLog2e;    // +inf: exp2(s - lse2) = 0
    cx.del = delta[(int64_t)head * d.nq + q_ld];
  }
  wait_vmem_all();

  const int64_t rel = d.q_off - d.kv_off;
  auto vis_count = [&](int i) -> int {
    if (!d.causal) return d.nkv;
    const int64_t v = (int64_t)i + rel + 1;
    return v <= 0 ? 0 : (v < d.nkv ? (int)v : d.nkv);
  };
  const int blk_last = min(q0 + DQ_ROWS, d.nq) - 1;
  const int nblk = (vis_count(blk_last) + BKS - 1) / BKS;
  const int w_first = min(q0 + wave * 32, d.nq - 1);
  const int w_last = min(q0 + wave * 32 + 31, d.nq - 1);
  const int nvis_wave = vis_count(w_last);
  const int nfull_wave = vis_count(w_first);
  cx.my_vis = vis_count(q_ld);
#pragma unroll
  for (int t = 0; t < 4; ++t) cx.dq[t] = zero16();

  cx.ka.init(lane, lds_base);
  cx.vnat = lds_base + DQ_VT + l32 * VT_LD + 16 * cx.half;

  // ---- staging, in two halves of 32 key rows so that only 16 registers are in flight: thread
  // moves chunk (tid & 15) of rows (tid >> 4) + 16 p of a half.  Rows beyond nkv re-read the last
  // row (finite values, masked out).
  const int st_row = tid >> 4, st_ch = tid & 15;
  u32x4 kreg[2], vreg[2];
  auto load_half = [&](int k0, int hf) {
    const gptr_t kb = uniform_gptr(K + (int64_t)k0 * H);
    const gptr_t vb = uniform_gptr(V + (int64_t)k0 * H);
    const int last = d.nkv - 1 - k0;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const unsigned off = (unsigned)(min(32 * hf + st_row + 16 * p, last) * (H * 2) + st_ch * 16);
      kreg[p] = gload_b128(kb, off);
      vreg[p] = gload_b128(vb, off);
    }
  };
  auto store_half = [&](int buf, int hf) {
    char* b = lds + buf * DQ_BUF;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int row = 32 * hf + st_row + 16 * p;
      *reinterpret_cast<u32x4*>(b + dual_store_off(row, st_ch)) = kreg[p];
      *reinterpret_cast<u32x4*>(b + DQ_VT + row * VT_LD + st_ch * 16) = vreg[p];
    }
  };

  if (nblk > 0) {
    load_half(0, 0); store_half(0, 0);
    load_half(0, 1); store_half(0, 1);
  }
  __syncthreads();

  for (int j = 0; j < nblk; ++j) {
    const int k0 = j * BKS;
    const bool more = j + 1 < nblk;
    if (more) load_half(k0 + BKS, 0);
    if (k0 < nvis_wave) {
      if (k0 + 32 > nfull_wave) dq_piece<0, true>(cx, k0); else dq_piece<0, false>(cx, k0);
    }
    if (more) { store_half((j + 1) & 1, 0); load_half(k0 + BKS, 1); }
    if (k0 + 32 < nvis_wave) {
      if (k0 + 64 > nfull_wave) dq_piece<1, true>(cx, k0 + 32); else dq_piece<1, false>(cx, k0 + 32);
    }
    if (more) store_half((j + 1) & 1, 1);
    const int tog = (j & 1) ? -DQ_BUF : DQ_BUF;
    cx.ka.shift(tog);
    cx.vnat += tog;
    __syncthreads();
  }
  if (q_ok) store_acc_t(dQ + ((int64_t)head * d.nq + q_row) * H, cx.dq, cx.half, d.scale);
}

}  // namespace

bool bwd_mfma_supported(const a2d_tile_desc& d) {
  return d.dtype == A2D_BF16 && d.hdim == mfma::H;
}

hipError_t launch_bwd_mfma(const a2d_tile_desc& d, const void* Q, const void* K, const void* V,
                           const void* dO, const float* lse, const float* delta, float* dQ,
                           float* dK, float* dV, hipStream_t s) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dkdv_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, DK_LDS);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_dq_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, DQ_LDS);
  if (e != hipSuccess) return e;
  dim3 grid_kv(xcd_grid(d.heads, (d.nkv + DK_KEYS - 1) / DK_KEYS));
  dim3 grid_q(xcd_grid(d.heads, (d.nq + DQ_ROWS - 1) / DQ_ROWS));
  hipLaunchKernelGGL(bwd_dkdv_kernel, grid_kv, dim3(DK_THREADS), DK_LDS, s, d, (const bf16_t*)Q,
                     (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dK, dV);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dq_kernel, grid_q, dim3(DQ_THREADS), DQ_LDS, s, d, (const bf16_t*)Q,
                     (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dQ);
  return hipGetLastError();
}

}  // namespace a2d
