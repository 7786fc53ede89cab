// bf16 MFMA backward tile kernels for H = 128, 96, 80 and 64: the per-tile gradient call of Alg. 3
// line 3 with P = exp(S - lse) rebuilt from the FINAL log-sum-exp of the query block,
//   dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = scale dS K,  dK = scale dS^T Q.
//
// Two kernels, so that every output has exactly one writer and no atomics are needed
// (bitwise reproducible results):
//   bwd_dkdv_kernel  owns key rows.  Workgroup = 8 wavefronts = 128 keys: four PAIRS of
//                    wavefronts (w, w + 4; both on SIMD w), 32 keys per pair.  The "score"
//                    wave of a pair holds the K^T fragments and the dV^T accumulators and
//                    computes S = Q K^T, P, dV^T += dO^T P; the "gradient" wave holds the V^T
//                    fragments and the dK^T accumulators and computes dP = dO V^T,
//                    dS = P o (dP - delta), dK^T += Q^T dS, with P handed over in fp32
//                    through LDS.  That halves the accumulators per wavefront (64 registers),
//                    so two wavefronts fit on a SIMD and one's exponentials overlap the
//                    other's MFMAs (a single wavefront cannot overlap the two).  The query
//                    blocks are walked 32 rows per step, staged through LDS together with dO,
//                    lse and delta; the gradient waves run one step behind the score waves, so
//                    one barrier per step is the only synchronisation.  S and dP leave a lane
//                    holding ONE key column, so P and dS feed the second contractions directly
//                    as B operands; dO^T / Q^T come from the LDS transpose read.
//   bwd_dq_kernel    owns query rows.  Workgroup = 8 wavefronts = 256 queries (32 per
//                    wavefront, Q and dO fragments in registers), two wavefronts per
//                    SIMD; walks the key blocks, 64 keys per step.  S^T = K Q^T
//                    and dP^T = V dO^T leave a lane holding ONE query column;
//                    dQ^T += K^T dS^T with K^T from the LDS transpose read.
//   bwd_dq_ds_kernel owns query rows like bwd_dq_kernel, but reads dS from a workspace the
//                    dK/dV kernel filled (its WRITE_DS variant) and only contracts it with K:
//                    used when the caller's workspace is large enough, so that S and dP are
//                    computed once (5 contractions for 5 counted ones instead of 7).
// Tiles that are read both ways (natural and transposed fragments) live in the "dual" LDS
// layout of a2d_mfma.hpp: every fragment address is a per-lane base plus an immediate.
#include <type_traits>

#include "a2d_mfma.hpp"

namespace a2d {
namespace {

using namespace mfma;

// stores a transposed accumulator (lane = one output row, registers = 4-column groups)
// (add: onto what the row already holds)
// CT column tiles of 32; pieces whose columns lie past the head size h are skipped
template <int CT>
__device__ __forceinline__ void store_acc_t(float* __restrict__ out_row, const f32x16 (&acc)[CT],
                                            int half, float mul, int h, bool add = false) {
#pragma unroll
  for (int ht = 0; ht < CT; ++ht)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (32 * ht + 8 * g + 4 * half >= h) continue;
      f32x4 v = {acc[ht][4 * g] * mul, acc[ht][4 * g + 1] * mul, acc[ht][4 * g + 2] * mul,
                 acc[ht][4 * g + 3] * mul};
      f32x4* p = reinterpret_cast<f32x4*>(out_row + 32 * ht + 8 * g + 4 * half);
      if (add) {
        const f32x4 o = *p;
        v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
      }
      *p = v;
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
constexpr int DK_THREADS = 512;
constexpr int DK_KEYS = 128;      // keys per workgroup
constexpr int BQ = 32;            // query rows per step
constexpr int DK_NBUF = 4;        // tile buffers: gradient waves' step, score waves' step, next, incoming
// LDS: [buf]{ Q tile, dO tile } (dual layout, 32 rows each) | [buf]{ lse*log2e [32], delta [32] } |
//      [slot][pair] probabilities handed from the score wave to the gradient wave (fp32)
constexpr int DK_TILE = BQ * DUAL_LD;
constexpr int DK_BUF = 2 * DK_TILE;
constexpr int DK_STAT = DK_NBUF * DK_BUF;
constexpr int DK_STAT_BUF = 2 * BQ * 4;
constexpr int DK_MBOX = DK_STAT + DK_NBUF * DK_STAT_BUF;
constexpr int DK_MBOX_PIECE = 32 * 32 * 4;
constexpr int DK_MBOX_SLOT = 4 * DK_MBOX_PIECE;
constexpr int DK_LDS = DK_MBOX + 2 * DK_MBOX_SLOT;

// Per-wavefront state.  The two roles run the same contraction code on different operands:
//   score wave (role 0):    frag = K^T fragments, natural reads from the Q tile,
//                           transposed reads from the dO tile, acc = dV^T
//   gradient wave (role 1): frag = V^T fragments, natural reads from the dO tile,
//                           transposed reads from the Q tile, acc = dK^T
template <int HD>
struct DkCtx {
  f32x16 acc[HD / 32];
  bf16x8 frag[HD / 16];
  unsigned nat_e, nat_o, tr_lo, tr_hi;   // dual-layout bases in the tile buffer of this wave's step
  unsigned stat;        // lse (role 0) or delta (role 1) row of that buffer, + 16 * half
  unsigned mbox;        // this lane's place in the pair's mailbox, slot of this wave's step
  float c;
  int my_first;         // first local query row that sees this lane's key
  int half;
};

// Fragment addresses inside the wave's tile buffer (per-lane base + immediate)
#define A2D_NAT(X) lds_load_b128((((X) & 1) ? cx.nat_o : cx.nat_e) + 64 * ((X) >> 1))
#define A2D_TR(U, HT) \
  lds_load_tr(cx.tr_lo + (U) * 16 * DUAL_LD + 64 * (HT), cx.tr_hi + (U) * 16 * DUAL_LD + 64 * (HT))
#define A2D_FENCE __builtin_amdgcn_sched_barrier(0);

// First contraction of a 32-query x 32-key step (S = Q K^T or dP = dO V^T): HD / 16 MFMAs over
// H.  The natural fragments travel through a ring of four: dk_first_pre requests fragments
// 0..3, the body requests the others while it consumes those.  (The fences keep the compiler
// from sinking the requests down to their uses.)
template <int HD>
__device__ __forceinline__ void dk_first_pre(const DkCtx<HD>& cx, bf16x8 (&n)[4]) {
  n[0] = A2D_NAT(0); n[1] = A2D_NAT(1); n[2] = A2D_NAT(2); n[3] = A2D_NAT(3);
  A2D_FENCE
}
// `init` is the starting value of the sum (zero for S, -delta for dP - delta).  Two accumulators
// (even / odd 16-wide slices of H): an MFMA that accumulates onto the result of the one issued
// just before it would wait for that result.
// KS: the slices that hold data (a head size of 80 fills five of the padded six)
template <int HD, int KS = HD / 16>
__device__ __forceinline__ f32x16 dk_first(const DkCtx<HD>& cx, bf16x8 (&n)[4], f32x16 init) {
  f32x16 sa = init, sb = zero16();
  static_for<0, KS>([&](auto X) {
    constexpr int x = decltype(X)::value;
    if constexpr (x & 1) sb = mma(n[x & 3], cx.frag[x], sb); else sa = mma(n[x & 3], cx.frag[x], sa);
    if constexpr (x + 4 < KS) { n[x & 3] = A2D_NAT(x + 4); A2D_FENCE }
  });
#pragma unroll
  for (int r = 0; r < 16; ++r) sa[r] += sb[r];
  return sa;
}

// The 32 per-query statistics of the step (lse for the score wave, delta for the gradient wave)
// and the partner's probabilities, requested ahead of the first contraction.
template <int HD>
__device__ __forceinline__ void dk_stat_pre(const DkCtx<HD>& cx, f32x4 (&st)[4]) {
#pragma unroll
  for (int g = 0; g < 4; ++g) st[g] = lds_load_f32x4(cx.stat + 8 * g * 4);
  A2D_FENCE
}
template <int HD>
__device__ __forceinline__ void dk_mbox_pre(const DkCtx<HD>& cx, f32x4 (&pm)[4]) {
#pragma unroll
  for (int g = 0; g < 4; ++g) pm[g] = lds_load_f32x4(cx.mbox + g * 1024);
  A2D_FENCE
}

// score wave: P = exp2(c S - lse2), masked; handed on in fp32 and kept as bf16 B fragments.
// register r <-> query qs0 + 8*(r>>2) + 4*half + (r&3); lane <-> key
template <bool MASK, int HD>
__device__ __forceinline__ void dk_probs(const DkCtx<HD>& cx, const f32x4 (&st)[4], f32x16& s,
                                         bf16x8 (&bf)[2], int qs0) {
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    f32x4 p4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float p = fast_exp2(fmaf(s[4 * g + e], cx.c, -st[g][e]));
      if (MASK && (qs0 + 8 * g + 4 * cx.half + e < cx.my_first)) p = 0.f;
      s[4 * g + e] = p;
      p4[e] = p;
    }
    *reinterpret_cast<__attribute__((address_space(3))) f32x4*>((uintptr_t)(cx.mbox + g * 1024)) = p4;
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) bf[u] = pack8(s, 8 * u);
}

// gradient wave: dS = P o (dP - delta) from the partner's probabilities; `dpd` is dP - delta
// already (the contraction started from -delta)
__device__ __forceinline__ void dk_dscores(const f32x4 (&pm)[4], f32x16& dpd, bf16x8 (&bf)[2]) {
  f32x16& dp = dpd;
#pragma unroll
  for (int g = 0; g < 4; ++g)
#pragma unroll
    for (int e = 0; e < 4; ++e) dp[4 * g + e] = pm[g][e] * dp[4 * g + e];
#pragma unroll
  for (int u = 0; u < 2; ++u) bf[u] = pack8(dp, 8 * u);
}

// Second contraction of a step (dV^T += dO^T P or dK^T += Q^T dS): 2 * HD / 32 MFMAs, A operands
// from the LDS transpose read, again through a ring (one fragment per 32-column tile of H):
// dk_second_pre requests those of the first 16 query rows (before the exponentials, so they
// arrive meanwhile), the body those of the second 16.
template <int HD>
__device__ __forceinline__ void dk_second_pre(const DkCtx<HD>& cx, bf16x8 (&t)[HD / 32]) {
  static_for<0, HD / 32>([&](auto HT) { constexpr int ht = decltype(HT)::value; t[ht] = A2D_TR(0, ht); });
  A2D_FENCE
}
template <int HD>
__device__ __forceinline__ void dk_second(DkCtx<HD>& cx, bf16x8 (&t)[HD / 32], const bf16x8 (&bf)[2]) {
  constexpr int CT = HD / 32;
  static_for<0, CT>([&](auto HT) {
    constexpr int ht = decltype(HT)::value;
    cx.acc[ht] = mma(t[ht], bf[0], cx.acc[ht]);
    t[ht] = A2D_TR(1, ht);
    A2D_FENCE
  });
  static_for<0, CT>([&](auto HT) {
    constexpr int ht = decltype(HT)::value;
    cx.acc[ht] = mma(t[ht], bf[1], cx.acc[ht]);
  });
}
#undef A2D_FENCE
#undef A2D_TR
#undef A2D_NAT

// ---- dS hand-over to the dQ kernel (optional).  The dK/dV kernel can leave dS (bf16, already
// multiplied out: P o (dP - delta)) in a workspace, so that the dQ kernel is a plain contraction
// dQ = scale dS K instead of recomputing S and dP.  Workspace layout: per head, per 32-row tile rt,
// per 64-key block kb one 4 KiB tile [piece T = 0, 1 (32 keys each)][u = 0, 1 (16 keys each)]
// [lane 0..63][8 bf16]: lane (row = lane & 31, half = lane >> 5) holds, for the 16 keys
// 64 kb + 32 T + 16 u + .., the keys 4 half + {0..3} and 8 + 4 half + {0..3} - exactly the B
// fragment of the dQ kernel's MFMA, so the consumer reads it with one coalesced 16-byte load per
// lane and the producer writes it with one coalesced 16-byte store per lane.
constexpr int DS_TILE_BYTES = 4096;
__host__ __device__ inline int ds_row_tiles(int nq) { return (nq + 31) / 32; }
__host__ __device__ inline int ds_key_blocks(int nkv) { return (nkv + 63) / 64; }
__host__ __device__ inline size_t ds_head_bytes(int nq, int nkv) {
  return (size_t)ds_row_tiles(nq) * ds_key_blocks(nkv) * DS_TILE_BYTES;
}

typedef __attribute__((address_space(1))) char* gwptr_t;
__device__ __forceinline__ gwptr_t uniform_gwptr(void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<gwptr_t>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void gstore_b128(gwptr_t base, unsigned byte_off, bf16x8 v) {
  // streamed once, read back by another kernel: keep it from displacing the Q / dO tiles in L2
  __builtin_nontemporal_store(v, reinterpret_cast<__attribute__((address_space(1))) bf16x8*>(base + byte_off));
}

// The gradient wave holds dS with lane = key and registers = query rows; the dQ kernel needs
// lane = query row and registers = keys.  The wave turns its 32 x 32 piece around through LDS (its
// own mailbox piece, free once the probabilities have been read): each lane writes its four
// 4-row groups as 8-byte pieces of a [key][row] tile (rows of 72 bytes: conflict-free), and the
// transposing read returns, per lane, four keys of one row.
constexpr int DS_TR_LD = 72;
__device__ __forceinline__ void ds_turn_write(unsigned piece, int l32, int half, const bf16x8 (&bf)[2]) {
  const unsigned a = piece + l32 * DS_TR_LD + 8 * half;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const u32x4 w = __builtin_bit_cast(u32x4, bf[u]);
    // register group g = 2u (w.x, w.y) and g = 2u + 1 (w.z, w.w): rows 8g + 4 half + 0..3
    *reinterpret_cast<__attribute__((address_space(3))) u32x2*>((uintptr_t)(a + 16 * (2 * u))) = u32x2{w[0], w[1]};
    *reinterpret_cast<__attribute__((address_space(3))) u32x2*>((uintptr_t)(a + 16 * (2 * u + 1))) = u32x2{w[2], w[3]};
  }
}
__device__ __forceinline__ void ds_turn_read(unsigned piece, int lane, bf16x8 (&out)[2]) {
  const int g16 = lane >> 4, j16 = lane & 15;
  const unsigned a = piece + (4 * (g16 >> 1) + (j16 >> 2)) * DS_TR_LD + (16 * (g16 & 1) + 4 * (j16 & 3)) * 2;
#pragma unroll
  for (int u = 0; u < 2; ++u) out[u] = lds_load_tr(a + 16 * u * DS_TR_LD, a + (16 * u + 8) * DS_TR_LD);
}

// HR: head size = row length in memory (80, 96 or 128); the LDS tiles and fragments are laid out
// for the padded head size HD = padded_head(HR) (96 or 128).
// GROUPED: several query heads per key/value head (g.group > 1); the plain kernel is compiled
// without the bookkeeping that walks them.
// WRITE_DS: the gradient waves also leave dS in the workspace `dS` (layout above) for the
// contraction-only dQ kernel.
// PLAIN: Q and dO are in the plain layout (row stride H, head stride nq * H): the staging offsets
// are then compile-time multiples and one offset serves both tensors (3 % on the recomputing path).
template <int HR, bool GROUPED, bool WRITE_DS, bool PLAIN = false>
__global__ __launch_bounds__(DK_THREADS) void bwd_dkdv_kernel(
    a2d_tile_desc d, SegList g, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ delta, float* __restrict__ dK, float* __restrict__ dV,
    bf16_t* __restrict__ dS) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
  int head, blk;
  // `head` is the KEY/VALUE head; its g.group query heads are consecutive rows of Q, dO, lse, delta.
  // With g.qsplit = Z > 1 (grouped heads only) Z workgroups share a key block: workgroup z walks the
  // query heads z * group / Z ... of the group and leaves its sums in partial buffer z (dK, dV then
  // point at Z buffers of [key/value heads][nkv][H], added up by a sum kernel afterwards).
  const int qsplit = GROUPED ? g.qsplit : 1;
  const int group = GROUPED ? g.group / qsplit : 1;          // query heads this workgroup walks
  int qh0 = 0;                                               // the first of them, as a head of Q
  {
    int unit;
    if (!xcd_map((GROUPED ? d.heads / g.group : d.heads) * qsplit, (d.nkv + DK_KEYS - 1) / DK_KEYS, g.by_size != 0,
                 unit, blk)) return;
    head = unit / qsplit;
    const int z = unit - head * qsplit;
    qh0 = GROUPED ? head * g.group + z * group : head;
    if (GROUPED && qsplit > 1) {
      const int64_t part = (int64_t)z * (d.heads / g.group) * d.nkv * HR;
      dK += part;
      dV += part;
    }
  }
  constexpr int HD = padded_head(HR), H = HR, KS = HD / 16, CT = HD / 32;
  constexpr int KSR = (HR + 15) / 16;       // slices of H that hold data
  const int k0 = blk * DK_KEYS;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int pair = wave & 3, role = wave >> 2;   // wavefronts w and w + 4 share 32 keys
  const int l32 = lane & 31;
  Q += (int64_t)qh0 * d.lq.head;
  dO += (int64_t)qh0 * d.ldo.head;
  K += (int64_t)head * d.lk.head;
  V += (int64_t)head * d.lv.head;
  lse += (int64_t)qh0 * d.nq;
  delta += (int64_t)qh0 * d.nq;

  DkCtx<HD> cx;
  cx.half = lane >> 5;
  cx.c = d.scale * kLog2e;
  // ---- K^T (score wave) or V^T (gradient wave) B fragments of the pair's 32 keys: lane = key,
  // h = 16 x + 8 half + 0..7.  Keys beyond nkv re-read the last key; the mask zeroes their
  // probabilities.
  const int key = k0 + pair * 32 + l32;
  {
    const bf16_t* src = (role ? V : K) + (int64_t)min(key, d.nkv - 1) * (role ? d.lv.row : d.lk.row) + 8 * cx.half;
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      if (16 * x < H) cx.frag[x] = *reinterpret_cast<const bf16x8*>(src + 16 * x);
      else cx.frag[x] = bf16x8{};                              // columns past the head size are zero
    }
  }
  wait_vmem_all();
#pragma unroll
  for (int t = 0; t < CT; ++t) cx.acc[t] = zero16();

  // Query i sees key kk of key/value sub-block s iff i >= kk - rel[s].  seg_first_row(sb, r): first
  // local query row that sees local key r of sub-block sb (nq if none does).
  auto seg_first_row = [&](int sb, int r) -> int {
    const int64_t f = (int64_t)(r - g.start[sb]) - g.rel[sb];
    return f <= 0 ? 0 : (f >= d.nq ? d.nq : (int)f);
  };
  // smallest / largest such row over the local keys a .. b - 1 (inside a sub-block it grows with
  // the key, so only the ends of the covered part of each sub-block matter).  Each sub-block's
  // table entries are read once, with no load depending on another.
  auto first_row_range = [&](int a, int b, int& lo, int& hi) {
    lo = d.nq; hi = 0;
    if (!d.causal) { lo = 0; return; }
    for (int sb = 0; sb < g.n; ++sb) {
      const int x = max(a, g.start[sb]), y = min(b, g.start[sb] + g.rows[sb]);
      if (x >= y) continue;
      lo = min(lo, seg_first_row(sb, x));
      hi = max(hi, seg_first_row(sb, y - 1));
    }
  };
  int wg_lo, wg_hi;
  first_row_range(k0, min(k0 + DK_KEYS, d.nkv), wg_lo, wg_hi);
  const int i_start = (wg_lo / BQ) * BQ;
  const int nsteps = (d.nq - i_start + BQ - 1) / BQ;   // steps per query head
  const int total = nsteps * group;                    // the group's query heads one after the other
  const int wk_first = k0 + pair * 32, wk_end = min(wk_first + 32, d.nkv);
  cx.my_first = d.nq;                                         // padding keys see nothing
  if (key < d.nkv) {
    cx.my_first = 0;
    if (d.causal) {
      for (int sb = 0; sb < g.n; ++sb)                        // uniform loop, per-lane select
        if (key >= g.start[sb] && key < g.start[sb] + g.rows[sb]) cx.my_first = seg_first_row(sb, key);
    }
  }
  int w_any = d.nq, w_all = d.nq;   // rows below w_any see none of the pair's keys, rows from w_all on all
  if (wk_first < wk_end) {
    first_row_range(wk_first, wk_end, w_any, w_all);
    if (wk_end < wk_first + 32) w_all = d.nq;                 // padding keys in the pair: always masked
  }

  // ---- The gradient waves run ONE STEP BEHIND the score waves: in iteration j the score wave
  // computes S, P, dV of step j and leaves P in mailbox slot j & 1, while the gradient wave of
  // the same SIMD computes dP, dS, dK of step j - 1 from slot (j - 1) & 1.  Inside an iteration
  // the two never wait for each other; the single barrier per iteration publishes the mailbox
  // and a tile.  Step s lives in tile buffer s % 4: during iteration j buffers (j - 1) % 4 and
  // j % 4 are being computed on, (j + 1) % 4 is complete already - so that every wave can
  // request the first fragments of its NEXT step before the barrier and start the following
  // iteration with its operands in registers - and (j + 2) % 4 is being filled.  The score wave
  // starts on buffer 0 / slot 0, the gradient wave one behind.
  {
    DualAddr a;
    a.init(lane, lds_base + (role ? (DK_NBUF - 1) * DK_BUF : 0));
    const unsigned nat_tile = role ? DK_TILE : 0, tr_tile = role ? 0 : DK_TILE;
    cx.nat_e = a.nat_e + nat_tile; cx.nat_o = a.nat_o + nat_tile;
    cx.tr_lo = a.tr_lo + tr_tile;  cx.tr_hi = a.tr_hi + tr_tile;
  }
  cx.stat = lds_base + DK_STAT + (role ? (DK_NBUF - 1) * DK_STAT_BUF + BQ * 4 : 0) + 16 * cx.half;
  cx.mbox = lds_base + DK_MBOX + (role ? DK_MBOX_SLOT : 0) + pair * DK_MBOX_PIECE + lane * 16;
  int cur = role ? DK_NBUF - 1 : 0;   // tile buffer of this wave's step

  // ---- staging of a 32-row step: thread moves chunk (tid & 15) of row (tid >> 4) of both tiles.
  // Global latency is longer than an iteration: step j + 4 is requested in iteration j and
  // written to LDS in iteration j + 2, through two register sets.  Rows beyond nq re-read the
  // last row; their lse entry is +inf, which makes exp2(s - lse) = 0 (also for rows whose lse is
  // -inf).  Steps beyond the last re-stage the last one (into a buffer nobody reads any more):
  // unconditional loads and stores keep the compiler's wait counters exact.
  static_assert(DK_THREADS == BQ * 16, "staging map: one 16-byte chunk of each tile per thread");
  const int st_row = tid >> 4, st_ch = tid & 15;
  const gptr_t q_base = uniform_gptr(Q), g_base = uniform_gptr(dO);
  const int st_off = dual_store_off(st_row, st_ch);
  u32x4 qreg[2], greg[2];
  float stat[2] = {0.f, 0.f};
  bool stat_ok[2] = {false, false};
  // (a chunk past the row's end - head sizes below 128 - re-reads the row's last chunk and is
  // stored as zeros or, past the padded head size, not at all: every lane issues every load)
  const int ld_ch = min(st_ch, H / 8 - 1);
  const bool ch_data = st_ch * 8 < H, ch_tile = st_ch * 8 < HD;
  // (load_step is called for steps 0, 1, 2, ... in order; with grouped heads ld_s / ld_row0 /
  // ld_left follow the next step's position - its step inside the query head, the head's first
  // row - without a division)
  // (ld_qh / ld_gh: byte offset of the query head's first row of Q / dO from the group's first head)
  int ld_s = 0, ld_row0 = 0, ld_left = total - 1;
  unsigned ld_qh = 0, ld_gh = 0;
  const unsigned q_row_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.lq.row * 2);
  const unsigned g_row_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.ldo.row * 2);
  const unsigned q_head_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.lq.head * 2);
  const unsigned g_head_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.ldo.head * 2);
  auto load_step = [&](int step, auto set_tag) {
    constexpr int SET = decltype(set_tag)::value;
    const int i0 = i_start + (GROUPED ? ld_s : min(step, nsteps - 1)) * BQ;
    if constexpr (PLAIN) {
      const unsigned off = (unsigned)((ld_row0 + min(i0 + st_row, d.nq - 1)) * (H * 2) + ld_ch * 16);
      qreg[SET] = gload_b128(q_base, off);
      greg[SET] = gload_b128(g_base, off);
    } else {
      const unsigned r = (unsigned)min(i0 + st_row, d.nq - 1);
      qreg[SET] = gload_b128(q_base, ld_qh + __umul24(r, q_row_bytes) + ld_ch * 16);
      greg[SET] = gload_b128(g_base, ld_gh + __umul24(r, g_row_bytes) + ld_ch * 16);
    }
    // raw statistic loads only: converting here would make the wave wait for everything just
    // issued.  Every thread loads one (only the first 64 values are used) so that each set is
    // the same number of loads in every wavefront.
    const int i = ld_row0 + min(i0 + (tid & (BQ - 1)), d.nq - 1);
    stat[SET] = (tid & BQ) ? delta[i] : lse[i];
    stat_ok[SET] = (i0 + (tid & (BQ - 1))) < d.nq;
    if constexpr (GROUPED) {   // next step; the last one repeats
      const bool more = ld_left > 0, wrap = ld_s + 1 == nsteps;
      ld_left -= more ? 1 : 0;
      ld_row0 += (more && wrap) ? d.nq : 0;
      ld_qh += (more && wrap) ? q_head_bytes : 0u;
      ld_gh += (more && wrap) ? g_head_bytes : 0u;
      ld_s = more ? (wrap ? 0 : ld_s + 1) : ld_s;
    }
  };
  auto store_step = [&](int buf, auto set_tag) {
    constexpr int SET = decltype(set_tag)::value;
    char* b = lds + buf * DK_BUF;
    if (HD == 128 || ch_tile) {
      const u32x4 zero = {0, 0, 0, 0};
      *reinterpret_cast<u32x4*>(b + st_off) = (HD == 128 || ch_data) ? qreg[SET] : zero;
      *reinterpret_cast<u32x4*>(b + DK_TILE + st_off) = (HD == 128 || ch_data) ? greg[SET] : zero;
    }
    if (tid < 2 * BQ) {
      float v = stat[SET];
      if (tid < BQ) v = (!stat_ok[SET] || v == -INFINITY) ? INFINITY : v * kLog2e;
      else v = stat_ok[SET] ? v : 0.f;
      reinterpret_cast<float*>(lds + DK_STAT + buf * DK_STAT_BUF)[tid] = v;
    }
  };
  using set0 = std::integral_constant<int, 0>;
  using set1 = std::integral_constant<int, 1>;

  if (nsteps > 0) {
    load_step(0, set0{}); load_step(1, set1{});
    store_step(0, set0{}); store_step(1, set1{});
    load_step(2, set0{}); load_step(3, set1{});
  }
  __syncthreads();

  // dS hand-over: this pair's 32 keys are piece T = pair & 1 of key block 2 blk + (pair >> 1)
  const unsigned ds_row_stride = (unsigned)ds_key_blocks(d.nkv) * DS_TILE_BYTES;
  const unsigned ds_lane_off = (unsigned)(2 * blk + (pair >> 1)) * DS_TILE_BYTES + (pair & 1) * 2048 + lane * 16;
  gwptr_t ds_base = nullptr;
  if constexpr (WRITE_DS)
    ds_base = uniform_gwptr(reinterpret_cast<char*>(dS) + (int64_t)qh0 * ds_head_bytes(d.nq, d.nkv));

  // A step is skipped (by both wavefronts of its pair) when none of its rows sees any of the
  // pair's keys; it is masked unless every row sees every key.
  // (step = position in the whole walk, s = its step inside its query head)
  // (rows past nq do not count: a pair without keys, w_any = nq, is never active - it has no
  // place in the dS workspace either)
  auto active = [&](int step, int s) {
    return step >= 0 && step < total && min(i_start + s * BQ + BQ - 1, d.nq - 1) >= w_any;
  };
  int cs = 0;                                                   // s of the iteration's step j
  auto next_s = [&](int s) { return (GROUPED && s + 1 == nsteps) ? 0 : s + 1; };
  int c_rt = i_start / BQ;                                      // dS row tile of step j, counted over the group's heads
  // (a head's steps end at its last row tile; the next head's start i_start / BQ tiles into its own)
  auto next_rt = [&](int rt, int s) { return (GROUPED && s + 1 == nsteps) ? rt + 1 + i_start / BQ : rt + 1; };
  auto advance = [&](int slot_delta) {   // to this wave's next step: tile buffer and mailbox slot
    const int adv = (cur == DK_NBUF - 1) ? -(DK_NBUF - 1) : 1;
    cur += adv;
    cx.nat_e += adv * DK_BUF; cx.nat_o += adv * DK_BUF; cx.tr_lo += adv * DK_BUF; cx.tr_hi += adv * DK_BUF;
    cx.stat += adv * DK_STAT_BUF;
    cx.mbox += slot_delta;
  };

  // The two roles go through an iteration in opposite phase, so that on every SIMD one wave's
  // element-wise work coincides with the other's MFMAs:
  //   score wave     S (8 MFMAs)          | exponentials          | dV (8 MFMAs)
  //   gradient wave  dS of step j - 1     | dK of step j - 1      | dP of step j (8 MFMAs each)
  // In iteration j, SET is the register set that holds step j + 2 and then receives step j + 4.
  if (nsteps > 0 && role == 0) {
    // first natural fragments and lse values of the coming step, requested an iteration ahead
    bf16x8 n[4];
    f32x4 st[4];
    dk_first_pre(cx, n);
    dk_stat_pre(cx, st);
    auto iteration = [&](int j, auto set_tag) {
      constexpr int SET = decltype(set_tag)::value;
      store_step((j + 2) % DK_NBUF, set_tag);
      load_step(j + 4, set_tag);
      if (active(j, cs)) {
        const int i0 = i_start + cs * BQ;
        bf16x8 t[CT], bf[2];
        f32x16 s = dk_first<HD, KSR>(cx, n, zero16());
        dk_second_pre(cx, t);
        if (i0 >= w_all && i0 + BQ <= d.nq) dk_probs<false>(cx, st, s, bf, i0);
        else dk_probs<true>(cx, st, s, bf, i0);
        dk_second(cx, t, bf);
      }
      advance(SET ? -DK_MBOX_SLOT : DK_MBOX_SLOT);
      cs = next_s(cs);
      dk_first_pre(cx, n);
      dk_stat_pre(cx, st);
      __syncthreads();
    };
    // nsteps + 1 iterations (the gradient wave's last step), rounded up to an even number: an
    // iteration beyond that finds no step to compute, and straight-line control flow keeps the
    // wait counters exact
    for (int j = 0; j <= total; j += 2) {
      iteration(j, set0{});
      iteration(j + 1, set1{});
    }
  } else if (nsteps > 0) {
    f32x16 dp = zero16();   // dP - delta of the step whose dS, dK come next iteration
    int ps = 0;             // s of step j - 1
    int p_rt = 0;           // and its dS row tile
    auto iteration = [&](int j, auto set_tag) {
      constexpr int SET = decltype(set_tag)::value;
      store_step((j + 2) % DK_NBUF, set_tag);
      load_step(j + 4, set_tag);
      if (active(j - 1, ps)) {
        bf16x8 t[CT], bf[2];
        f32x4 pm[4];
        dk_mbox_pre(cx, pm);
        dk_second_pre(cx, t);
        dk_dscores(pm, dp, bf);
        bf16x8 ds_out[2];
        if constexpr (WRITE_DS) {
          // turned around through LDS; requested BEFORE the contraction's own fragments are
          // waited for (LDS answers in order), so the stores below find their data arrived
          ds_turn_write(cx.mbox - lane * 16, l32, cx.half, bf);
          ds_turn_read(cx.mbox - lane * 16, lane, ds_out);
          __builtin_amdgcn_sched_barrier(0);
        }
        dk_second(cx, t, bf);
        if constexpr (WRITE_DS) {
          // (measured: making these stores unconditional - skipped steps writing to a spill slot,
          // which keeps the compiler's load wait counts exact - is not faster)
          const unsigned off = (unsigned)p_rt * ds_row_stride + ds_lane_off;
          gstore_b128(ds_base, off, ds_out[0]);
          gstore_b128(ds_base, off + 1024, ds_out[1]);
        }
      }
      advance(SET ? DK_MBOX_SLOT : -DK_MBOX_SLOT);
      p_rt = c_rt;
      c_rt = next_rt(c_rt, cs);
      ps = cs;
      cs = next_s(cs);
      if (active(j, ps)) {
        bf16x8 n[4];
        f32x4 st[4];
        dk_first_pre(cx, n);
        dk_stat_pre(cx, st);
        f32x16 init;
#pragma unroll
        for (int r = 0; r < 16; ++r) init[r] = -st[r >> 2][r & 3];
        dp = dk_first<HD, KSR>(cx, n, init);
      }
      __syncthreads();
    };
    for (int j = 0; j <= total; j += 2) {
      iteration(j, set0{});
      iteration(j + 1, set1{});
    }
  }

  if (key < d.nkv) {
    const int64_t row = (int64_t)head * d.nkv + key;
    if (role == 0) store_acc_t<CT>(dV + row * H, cx.acc, cx.half, 1.0f, H);
    else store_acc_t<CT>(dK + row * H, cx.acc, cx.half, d.scale, H);
  }
}

// ---------------------------------------------------------------------- dQ
constexpr int BKS = 64;           // keys per step
// LDS: [buf]{ K tile (dual layout), V tile (natural reads only: rows of the head's bytes + 16) }
__host__ __device__ constexpr int vt_ld(int hd) { return hd * 2 + 16; }
constexpr int DQ_VT = DUAL64_BYTES;
__host__ __device__ constexpr int dq_buf(int hd) { return DUAL64_BYTES + BKS * vt_ld(hd); }
__host__ __device__ constexpr int dq_lds(int hd) { return 2 * dq_buf(hd); }
constexpr int DQ_RING = 2;        // fragment ring depth (registers are tight: 256 per wavefront)

template <int HD>
struct DqCtx {
  f32x16 dq[HD / 32];
  bf16x8 qf[HD / 16], gf[HD / 16];
  DualAddr ka;          // K tile of the current buffer
  unsigned vnat;        // natural-fragment base in the V tile of the current buffer
  float c, lse2, del;
  int my_vis;           // number of leading local keys this lane's query row sees
  int half;
};

// one 32-key x 32-query piece: T selects the half of the 64-key step.  HD / 16 slices of H in the
// two first contractions (S^T and dP^T, alternating), 2 * HD / 32 MFMAs in dQ^T += K^T dS^T
// (step I: 16-key group I / CT, column tile I % CT); fragments run two steps ahead of their use.
// (KS: the slices that hold data - a head size of 80 fills five of the padded six)
template <int T, bool MASK, int HD, int KS = HD / 16>
__device__ __forceinline__ void dq_piece(DqCtx<HD>& cx, int key0) {
  constexpr int CT = HD / 32, VT_LD = vt_ld(HD);
  constexpr int RB = T * 32 * DUAL_LD;
  constexpr int VB = T * 32 * VT_LD;
  bf16x8 kr[DQ_RING], vr[DQ_RING], kt[DQ_RING];
  auto ld1 = [&](auto X) {
    constexpr int x = decltype(X)::value;
    kr[x % DQ_RING] = dual_nat<x>(cx.ka, RB);
    vr[x % DQ_RING] = lds_load_b128(cx.vnat + VB + 32 * x);
    __builtin_amdgcn_sched_barrier(0);
  };
  // K^T fragments; the first ones are on their way during the exponentials
  auto ld2 = [&](auto I) {
    constexpr int i = decltype(I)::value;
    kt[i % DQ_RING] = lds_load_tr(cx.ka.tr_lo + RB + (i / CT) * 16 * DUAL_LD + 64 * (i % CT),
                                  cx.ka.tr_hi + RB + (i / CT) * 16 * DUAL_LD + 64 * (i % CT));
    __builtin_amdgcn_sched_barrier(0);
  };
  static_for<0, DQ_RING>(ld1);
  f32x16 s = zero16(), dp = zero16();
  static_for<0, KS>([&](auto X) {
    constexpr int x = decltype(X)::value;
    s = mma(kr[x % DQ_RING], cx.qf[x], s);
    dp = mma(vr[x % DQ_RING], cx.gf[x], dp);
    if constexpr (x + DQ_RING < KS) ld1(std::integral_constant<int, x + DQ_RING>{});
    else ld2(std::integral_constant<int, x + DQ_RING - KS>{});
  });
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
  static_for<0, 2 * CT>([&](auto I) {
    constexpr int i = decltype(I)::value;
    cx.dq[i % CT] = mma(kt[i % DQ_RING], dsb[i / CT], cx.dq[i % CT]);
    if constexpr (i + DQ_RING < 2 * CT) ld2(std::integral_constant<int, i + DQ_RING>{});
  });
}

// WAVES wavefronts (32 query rows each) per workgroup: 8 fill a compute unit with one workgroup;
// 4 (two workgroups per compute unit) are used when there are too few 256-row blocks to give
// every compute unit one.
// KL key lanes of WAVES / KL wavefronts: with KL = 2 a 128-row workgroup of eight wavefronts walks
// the key blocks in two lanes (alternate blocks, own tile buffers) whose dQ sums are added through
// LDS at the end - for tiles with at most one 128-row block per compute unit, so that a SIMD still
// holds two wavefronts.
// HR: head size (80, 96 or 128), HD its padded size, as in the dK/dV kernel.
template <int WAVES, int HR, int KL>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void bwd_dq_kernel(
    a2d_tile_desc d, SegList g, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ delta, float* __restrict__ dQ) {
  extern __shared__ __attribute__((aligned(1024))) char lds_all[];
  constexpr int RW = WAVES / KL;           // wavefronts of one key lane
  constexpr int DQ_ROWS = 32 * RW;         // query rows per workgroup
  constexpr int DQ_THREADS = 64 * RW;      // threads of one key lane (they stage its tiles)
  constexpr int HD = padded_head(HR), H = HR;
  constexpr int KS = HD / 16, CT = HD / 32, VT_LD = vt_ld(HD), DQ_BUF = dq_buf(HD);
  constexpr int KSR = (HR + 15) / 16;      // slices of H that hold data
  const int kl = KL == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / DQ_THREADS);
  char* const lds = lds_all + kl * (2 * DQ_BUF);
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
  const int nqb = (d.nq + DQ_ROWS - 1) / DQ_ROWS;
  // the query blocks of the query heads that share a key/value head go to one XCD (to g.split
  // XCDs, an equal share of the heads each, when that is what spreads the load evenly)
  int unit, blk;
  const int per_unit = g.group / g.split;
  if (!xcd_map(d.heads / per_unit, per_unit * nqb, g.by_size != 0, unit, blk)) return;
  // (blocks numbered by size first when the workgroups are ordered by size)
  const int head = unit * per_unit + (g.by_size ? blk % per_unit : blk / nqb), kvh = head / g.group;
  blk = g.by_size ? blk / per_unit : blk % nqb;
  const int q0 = (nqb - 1 - blk) * DQ_ROWS;            // heavy blocks first under a causal mask
  const int tid = (int)threadIdx.x - kl * DQ_THREADS;  // within the key lane
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31;
  Q += (int64_t)head * d.lq.head;
  dO += (int64_t)head * d.ldo.head;
  K += (int64_t)kvh * d.lk.head;
  V += (int64_t)kvh * d.lv.head;

  DqCtx<HD> cx;
  cx.half = lane >> 5;
  cx.c = d.scale * kLog2e;
  const int q_row = q0 + wave * 32 + l32;
  const bool q_ok = q_row < d.nq;
  const int q_ld = min(q_row, d.nq - 1);         // rows beyond nq re-read the last row, lse2 = +inf
  {
    const int64_t off = (int64_t)q_ld * d.lq.row + 8 * cx.half, goff = (int64_t)q_ld * d.ldo.row + 8 * cx.half;
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      if (16 * x < H) {
        cx.qf[x] = *reinterpret_cast<const bf16x8*>(Q + off + 16 * x);
        cx.gf[x] = *reinterpret_cast<const bf16x8*>(dO + goff + 16 * x);
      } else {                                                 // columns past the head size are zero
        cx.qf[x] = bf16x8{};
        cx.gf[x] = bf16x8{};
      }
    }
    const float v = lse[(int64_t)head * d.nq + q_ld];
    cx.lse2 = (!q_ok || v == -INFINITY) ? INFINITY : v * kLog2e;    // +inf: exp2(s - lse2) = 0
    cx.del = delta[(int64_t)head * d.nq + q_ld];
  }
  wait_vmem_all();

  // visibility per key/value sub-block s: query i sees the first vis_count(i, s) keys of it
  auto vis_count = [&](int i, int s) -> int {
    if (!d.causal) return g.rows[s];
    const int64_t v = (int64_t)i + g.rel[s] + 1;
    return v <= 0 ? 0 : (v < g.rows[s] ? (int)v : g.rows[s]);
  };
  const int blk_last = min(q0 + DQ_ROWS, d.nq) - 1;
  const int w_first = min(q0 + wave * 32, d.nq - 1);
  const int w_last = min(q0 + wave * 32 + 31, d.nq - 1);
  // key blocks of sub-block s that some row of the workgroup sees; the walk over (sub-block, block)
  auto seg_blocks = [&](int s) { return (vis_count(blk_last, s) + BKS - 1) / BKS; };
  int nvis_wave = 0, nfull_wave = 0;               // of the current sub-block
  auto enter_segment = [&](int s) {
    nvis_wave = vis_count(w_last, s);
    nfull_wave = vis_count(w_first, s);
    cx.my_vis = vis_count(q_ld, s);
  };
#pragma unroll
  for (int t = 0; t < CT; ++t) cx.dq[t] = zero16();

  cx.ka.init(lane, lds_base);
  cx.vnat = lds_base + DQ_VT + l32 * VT_LD + 16 * cx.half;

  // ---- staging, in two halves of 32 key rows: thread moves chunk (tid & 15) of rows
  // (tid >> 4) + ST_ROWS p of a half.  Rows beyond nkv re-read the last row (finite values,
  // masked out).
  constexpr int ST_ROWS = DQ_THREADS / 16, ST_N = 32 / ST_ROWS;
  const int st_row = tid >> 4, st_ch = tid & 15;
  u32x4 kreg[ST_N], vreg[ST_N];
  // half hf of block j of the sub-block of seg_rows keys that starts at local key seg_start
  // (a chunk past the row's end - head sizes below 128 - re-reads the row's last chunk and is
  // stored as zeros or, past the padded head size, not at all)
  const int ld_ch = min(st_ch, H / 8 - 1);
  const bool ch_data = st_ch * 8 < H, ch_tile = st_ch * 8 < HD;
  // (row strides in bytes, pinned in registers: read from the kernel arguments inside the loop they
  // would be scalar loads, which share a wait counter with the LDS reads in flight.  A head's rows
  // span less than 4 GiB - the API layer checks it - so row index times stride fits 32 bits.)
  const unsigned k_row_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.lk.row * 2);
  const unsigned v_row_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.lv.row * 2);
  auto load_half = [&](int seg_start, int seg_rows, int j, int hf) {
    const int k0 = seg_start + j * BKS;
    const gptr_t kb = uniform_gptr(reinterpret_cast<const char*>(K) + (unsigned)k0 * k_row_bytes);
    const gptr_t vb = uniform_gptr(reinterpret_cast<const char*>(V) + (unsigned)k0 * v_row_bytes);
    const int last = seg_rows - 1 - j * BKS;       // rows beyond the sub-block re-read its last row
#pragma unroll
    for (int p = 0; p < ST_N; ++p) {
      const unsigned r = (unsigned)min(32 * hf + st_row + ST_ROWS * p, last);
      kreg[p] = gload_b128(kb, __umul24(r, k_row_bytes) + ld_ch * 16);
      vreg[p] = gload_b128(vb, __umul24(r, v_row_bytes) + ld_ch * 16);
    }
  };
  auto store_half = [&](int buf, int hf) {
    char* b = lds + buf * DQ_BUF;
    if (HD == 128 || ch_tile) {
      const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
      for (int p = 0; p < ST_N; ++p) {
        const int row = 32 * hf + st_row + ST_ROWS * p;
        *reinterpret_cast<u32x4*>(b + dual_store_off(row, st_ch)) = (HD == 128 || ch_data) ? kreg[p] : zero;
        *reinterpret_cast<u32x4*>(b + DQ_VT + row * VT_LD + st_ch * 16) = (HD == 128 || ch_data) ? vreg[p] : zero;
      }
    }
  };

  // Walk over the entries (sub-block, key block); key lane kl takes entries kl, kl + KL, ...  The
  // sub-block table lives in kernel-argument memory, and scalar loads share a wait counter with the
  // LDS reads in flight, so it is only touched when a walk moves to another sub-block; in between
  // its values sit in registers.  An entry is (sub-block sb, block j of its nblk); sb == g.n: past
  // the end.
  auto open_segment = [&](int s, int& sb, int& j, int& nblk) {   // first sub-block after s with visible keys
    do { ++s; } while (s < g.n && seg_blocks(s) == 0);
    sb = s; j = 0;
    if (s < g.n) nblk = seg_blocks(s);
  };
  auto advance = [&](int& sb, int& j, int& nblk) {
    if (sb < g.n && ++j >= nblk) open_segment(sb, sb, j, nblk);
  };
  int sb, j, nblk = 0;                             // this key lane's current entry
  open_segment(-1, sb, j, nblk);
  int lead_sb = sb, lead_j = j, lead_nblk = nblk;  // key lane 0's: every lane loops while it exists
  if (KL > 1) {
    for (int x = 0; x < kl; ++x) advance(sb, j, nblk);
  }
  int nx_start = 0, nx_rows = 0;                   // start / rows of the next entry's sub-block
  if (sb < g.n) {
    enter_segment(sb);
    nx_start = g.start[sb]; nx_rows = g.rows[sb];
    load_half(nx_start, nx_rows, j, 0); store_half(0, 0);
    load_half(nx_start, nx_rows, j, 1); store_half(0, 1);
  }
  __syncthreads();

  int buf = 0;
  while ((KL == 1 ? sb : lead_sb) < g.n) {
    int nsb = sb, nj = j, nnblk = nblk;
#pragma unroll
    for (int x = 0; x < KL; ++x) advance(nsb, nj, nnblk);
    const bool more = nsb < g.n;
    if (more && nsb != sb) { nx_start = g.start[nsb]; nx_rows = g.rows[nsb]; }
    const bool here = KL == 1 || sb < g.n;         // this lane has a block in this round
    const int k0 = j * BKS;                        // local to the sub-block
    if (more) load_half(nx_start, nx_rows, nj, 0);
    if (here && k0 < nvis_wave) {
      if (k0 + 32 > nfull_wave) dq_piece<0, true, HD, KSR>(cx, k0); else dq_piece<0, false, HD, KSR>(cx, k0);
    }
    if (more) { store_half(buf ^ 1, 0); load_half(nx_start, nx_rows, nj, 1); }
    if (here && k0 + 32 < nvis_wave) {
      if (k0 + 64 > nfull_wave) dq_piece<1, true, HD, KSR>(cx, k0 + 32); else dq_piece<1, false, HD, KSR>(cx, k0 + 32);
    }
    if (more) store_half(buf ^ 1, 1);
    const int tog = buf ? -DQ_BUF : DQ_BUF;
    cx.ka.shift(tog);
    cx.vnat += tog;
    __syncthreads();
    if (more && nsb != sb) enter_segment(nsb);
    if (KL > 1) {
#pragma unroll
      for (int x = 0; x < KL; ++x) advance(lead_sb, lead_j, lead_nblk);
    }
    sb = nsb; j = nj; nblk = nnblk;
    buf ^= 1;
  }
  if constexpr (KL == 2) {
    // lane 1 hands its sums to lane 0 through LDS (the tiles are no longer read: every wavefront
    // has passed the walk's last barrier); layout [row wavefront][value][lane]: conflict free
    static_assert(RW * CT * 16 * 256 <= KL * 2 * DQ_BUF, "the exchange area must fit the tile buffers");
    float* xch = reinterpret_cast<float*>(lds_all) + wave * (CT * 16 * 64) + lane;
    if (kl == 1) {
#pragma unroll
      for (int t = 0; t < CT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) xch[(16 * t + r) * 64] = cx.dq[t][r];
    }
    __syncthreads();
    if (kl == 1) return;
#pragma unroll
    for (int t = 0; t < CT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) cx.dq[t][r] += xch[(16 * t + r) * 64];
  }
  if (q_ok) store_acc_t<CT>(dQ + ((int64_t)head * d.nq + q_row) * H, cx.dq, cx.half, d.scale, H, g.acc != 0);
}

// ---------------------------------------------------------------------- dQ from a stored dS
// Contraction-only dQ kernel: dQ^T += K^T dS^T with dS read back from the workspace the dK/dV
// kernel filled (layout at ds_row_tiles above).  Workgroup = WAVES wavefronts of 32 query rows;
// 64 keys per step: the K tile goes through LDS (dual layout, transposing reads only), the dS
// fragments come straight from global memory, one contiguous 4 KiB tile per wavefront and step,
// requested DSQ_SETS - 1 steps ahead through DSQ_SETS register sets (the stream is HBM-bound: 2 bytes per
// score).  The sub-blocks of a gathered tile must start at multiples of 64 keys, so that a 64-key
// block never straddles two of them.
constexpr int DSQ_RING = 4;
constexpr int DSQ_SETS = 3;  // register sets of dS fragments: requests run DSQ_SETS - 1 steps ahead
template <int HD>
struct DsqCtx {
  f32x16 dq[HD / 32];
  DualAddr ka;          // K tile of the current buffer
  int my_vis;           // number of leading keys of the current sub-block this lane's query row sees
  int half;
};

// one 32-key piece (T = 0, 1) of the step: ds[2T], ds[2T + 1] are the two 16-key B fragments;
// key0 = the piece's first key, local to its sub-block
template <int T, bool MASK, int HD>
__device__ __forceinline__ void dsq_piece(DsqCtx<HD>& cx, const u32x4 (&ds)[4], int key0) {
  constexpr int CT = HD / 32;
  constexpr int RB = T * 32 * DUAL_LD;
  bf16x8 kt[DSQ_RING];
  auto ld = [&](auto I) {
    constexpr int i = decltype(I)::value;
    kt[i % DSQ_RING] = lds_load_tr(cx.ka.tr_lo + RB + (i / CT) * 16 * DUAL_LD + 64 * (i % CT),
                                   cx.ka.tr_hi + RB + (i / CT) * 16 * DUAL_LD + 64 * (i % CT));
    __builtin_amdgcn_sched_barrier(0);
  };
  static_for<0, (DSQ_RING < 2 * CT ? DSQ_RING : 2 * CT)>(ld);
  bf16x8 dsb[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    u32x4 w = ds[2 * T + u];
    if (MASK) {
      // element e of the fragment <-> key key0 + 16u + 8 (e >> 2) + 4 half + (e & 3); two per word
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int k = key0 + 16 * u + 8 * (x >> 1) + 4 * cx.half + 2 * (x & 1);
        const unsigned keep = (k < cx.my_vis ? 0x0000FFFFu : 0u) | (k + 1 < cx.my_vis ? 0xFFFF0000u : 0u);
        w[x] &= keep;
      }
    }
    dsb[u] = __builtin_bit_cast(bf16x8, w);
  }
  static_for<0, 2 * CT>([&](auto I) {
    constexpr int i = decltype(I)::value;
    cx.dq[i % CT] = mma(kt[i % DSQ_RING], dsb[i / CT], cx.dq[i % CT]);
    if constexpr (i + DSQ_RING < 2 * CT) ld(std::integral_constant<int, i + DSQ_RING>{});
  });
}

// KL key lanes of WAVES / KL wavefronts: with KL = 2 a 128-row workgroup of eight wavefronts walks
// the key blocks in two lanes (alternate blocks, own K buffers) whose dQ sums are added through LDS
// at the end - for tiles with at most one 128-row block per compute unit, so that a SIMD still
// holds two wavefronts and twice the dS requests are in flight.
template <int WAVES, int HR, int KL>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void bwd_dq_ds_kernel(
    a2d_tile_desc d, SegList g, const bf16_t* __restrict__ K, const bf16_t* __restrict__ dS,
    float* __restrict__ dQ) {
  extern __shared__ __attribute__((aligned(1024))) char lds_all[];
  constexpr int RW = WAVES / KL;                       // wavefronts of one key lane
  constexpr int DQ_ROWS = 32 * RW, DQ_THREADS = 64 * RW;   // rows of the workgroup, threads of one key lane
  const int kl = KL == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / DQ_THREADS);
  char* const lds = lds_all + kl * (2 * DUAL64_BYTES);
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
  constexpr int HD = padded_head(HR), H = HR, CT = HD / 32;
  const int nqb = (d.nq + DQ_ROWS - 1) / DQ_ROWS;
  // placement as in bwd_dq_kernel (grouped heads: the query heads of a key/value head share an XCD)
  int unit, blk;
  const int per_unit = g.group / g.split;
  if (!xcd_map(d.heads / per_unit, per_unit * nqb, g.by_size != 0, unit, blk)) return;
  // (blocks numbered by size first when the workgroups are ordered by size)
  const int head = unit * per_unit + (g.by_size ? blk % per_unit : blk / nqb), kvh = head / g.group;
  blk = g.by_size ? blk / per_unit : blk % nqb;
  const int q0 = (nqb - 1 - blk) * DQ_ROWS;            // heavy blocks first under a causal mask
  const int tid = (int)threadIdx.x - kl * DQ_THREADS;  // within the key lane
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31;
  K += (int64_t)kvh * d.lk.head;

  DsqCtx<HD> cx;
  cx.half = lane >> 5;
  const int q_row = q0 + wave * 32 + l32;
  const bool q_ok = q_row < d.nq;
  const int q_ld = min(q_row, d.nq - 1);
#pragma unroll
  for (int t = 0; t < CT; ++t) cx.dq[t] = zero16();
  cx.ka.init(lane, lds_base);

  // this wavefront's row tile of dS (a wavefront past the last row reads the last tile; its
  // results are never stored)
  const int n_rt = ds_row_tiles(d.nq), n_kb = ds_key_blocks(d.nkv);
  const int rt = min((q0 + wave * 32) / 32, n_rt - 1);
  const gptr_t ds_base = uniform_gptr(reinterpret_cast<const char*>(dS) + (int64_t)head * ds_head_bytes(d.nq, d.nkv) +
                                      (int64_t)rt * n_kb * DS_TILE_BYTES);

  // visibility per key/value sub-block s: query i sees the first vis_count(i, s) keys of it
  auto vis_count = [&](int i, int s) -> int {
    if (!d.causal) return g.rows[s];
    const int64_t v = (int64_t)i + g.rel[s] + 1;
    return v <= 0 ? 0 : (v < g.rows[s] ? (int)v : g.rows[s]);
  };
  const int blk_last = min(q0 + DQ_ROWS, d.nq) - 1;
  const int w_first = min(q0 + wave * 32, d.nq - 1);
  const int w_last = min(q0 + wave * 32 + 31, d.nq - 1);
  auto seg_blocks = [&](int s) { return (vis_count(blk_last, s) + BKS - 1) / BKS; };
  int count = 0;                                   // 64-key blocks the workgroup walks
  for (int s = 0; s < g.n; ++s) count += seg_blocks(s);

  // Walk over the visible blocks, as global block numbers (start of the sub-block / 64 + block
  // inside it).  The fetch walker runs ahead of the compute walker; once it has run out it keeps
  // returning its last block (loads stay unconditional).
  // (a key lane takes every KL-th block: each walker moves KL blocks per call, after kl at the start)
  int f_sb = -1, f_j = 0, f_nblk = 0, f_base = 0, f_id = 0;
  auto fetch_one = [&]() {
    if (f_j + 1 < f_nblk) { ++f_j; f_id = f_base + f_j; return; }
    int s = f_sb + 1;
    while (s < g.n && seg_blocks(s) == 0) ++s;
    if (s < g.n) { f_sb = s; f_j = 0; f_nblk = seg_blocks(s); f_base = g.start[s] / BKS; f_id = f_base; }
  };
  auto fetch_next = [&]() {
#pragma unroll
    for (int x = 0; x < KL; ++x) fetch_one();
  };
  int c_sb = -1, c_j = 0, c_nblk = 0;              // compute walker: sub-block, block inside it
  int nvis_wave = 0, nfull_wave = 0;
  auto compute_one = [&]() {
    if (c_j + 1 < c_nblk) { ++c_j; return; }
    int s = c_sb + 1;
    while (s < g.n && seg_blocks(s) == 0) ++s;
    if (s < g.n) {
      c_sb = s; c_j = 0; c_nblk = seg_blocks(s);
      nvis_wave = vis_count(w_last, s);
      nfull_wave = vis_count(w_first, s);
      cx.my_vis = vis_count(q_ld, s);
    } else {
      nvis_wave = 0;                               // past the last block: nothing to compute
    }
  };
  auto compute_next = [&]() {
#pragma unroll
    for (int x = 0; x < KL; ++x) compute_one();
  };

  // ---- K staging: thread moves chunk (tid & 15) of rows (tid >> 4) + ST_ROWS p of the 64-row tile
  constexpr int ST_ROWS = DQ_THREADS / 16, ST_N = BKS / ST_ROWS;
  const int st_row = tid >> 4, st_ch = tid & 15;
  const int ld_ch = min(st_ch, H / 8 - 1);
  const bool ch_data = st_ch * 8 < H, ch_tile = st_ch * 8 < HD;
  const gptr_t k_base = uniform_gptr(K);
  const unsigned k_row_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.lk.row * 2);
  u32x4 kreg[ST_N];
  auto load_k = [&](int id) {
#pragma unroll
    for (int p = 0; p < ST_N; ++p) {
      const int row = min(id * BKS + st_row + ST_ROWS * p, d.nkv - 1);   // rows past the end re-read the last key
      kreg[p] = gload_b128(k_base, __umul24((unsigned)row, k_row_bytes) + ld_ch * 16);
    }
  };
  auto store_k = [&](int buf) {
    char* b = lds + buf * DUAL64_BYTES;
    if (HD == 128 || ch_tile) {
      const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
      for (int p = 0; p < ST_N; ++p)
        *reinterpret_cast<u32x4*>(b + dual_store_off(st_row + ST_ROWS * p, st_ch)) = (HD == 128 || ch_data) ? kreg[p] : zero;
    }
  };
  u32x4 ds[DSQ_SETS][4];
  auto load_ds = [&](int id, auto set_tag) {
    constexpr int SET = decltype(set_tag)::value;
    const unsigned off = (unsigned)id * DS_TILE_BYTES + lane * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // read once: keep the stream from displacing the K tiles in L2
      ds[SET][i] = __builtin_nontemporal_load(
          reinterpret_cast<const __attribute__((address_space(1))) u32x4*>(ds_base + off + 1024 * i));
    }
  };

  if (count == 0) {                                // no visible key: dQ share is zero
    if (q_ok && !g.acc && kl == 0) store_acc_t<CT>(dQ + ((int64_t)head * d.nq + q_row) * H, cx.dq, cx.half, 0.f, H, false);
    return;
  }
  if (KL > 1) {
    for (int x = 0; x < kl; ++x) { fetch_one(); compute_one(); }
    fetch_one();                                   // this lane's first block (the last one, if it has none)
  } else {
    fetch_next();                                  // block 0
  }
  load_k(f_id);
  load_ds(f_id, std::integral_constant<int, 0>{});
  store_k(0);
  int idq[DSQ_SETS - 2];                           // blocks t + 1 .. t + DSQ_SETS - 2 of iteration t
  static_for<1, DSQ_SETS - 1>([&](auto S) {        // blocks 1 .. DSQ_SETS - 2
    fetch_next();
    idq[decltype(S)::value - 1] = f_id;
    load_ds(f_id, S);
  });
  if (KL > 1) compute_one(); else compute_next();
  __syncthreads();

  int buf = 0;
  // iteration t: K of block t + 1 and dS of block t + DSQ_SETS - 1 are requested (K first: the
  // wait for it at the end of the iteration must not cover the dS loads behind it), block t is
  // computed.
  auto iteration = [&](auto cur_tag) {
    constexpr int CUR = decltype(cur_tag)::value;
    load_k(idq[0]);
    fetch_next();
    load_ds(f_id, std::integral_constant<int, (CUR + DSQ_SETS - 1) % DSQ_SETS>{});
    const int k0 = c_j * BKS;                      // local to the sub-block
    if (k0 < nvis_wave) {
      if (k0 + 32 > nfull_wave) dsq_piece<0, true>(cx, ds[CUR], k0); else dsq_piece<0, false>(cx, ds[CUR], k0);
    }
    if (k0 + 32 < nvis_wave) {
      if (k0 + 64 > nfull_wave) dsq_piece<1, true>(cx, ds[CUR], k0 + 32); else dsq_piece<1, false>(cx, ds[CUR], k0 + 32);
    }
    store_k(buf ^ 1);
#pragma unroll
    for (int x = 0; x + 1 < DSQ_SETS - 2; ++x) idq[x] = idq[x + 1];
    idq[DSQ_SETS - 3] = f_id;
    cx.ka.shift(buf ? -DUAL64_BYTES : DUAL64_BYTES);
    buf ^= 1;
    compute_next();
    __syncthreads();
  };
  for (int t = 0; t < (count + KL - 1) / KL; t += DSQ_SETS)   // blocks past the last find nvis_wave = 0
    static_for<0, DSQ_SETS>([&](auto S) { iteration(S); });
  if constexpr (KL == 2) {
    // lane 1 hands its sums to lane 0 through LDS (the K tiles are no longer read: every wavefront
    // has passed the walk's last barrier); layout [row wavefront][value][lane]: conflict free
    static_assert(RW * CT * 16 * 256 <= KL * 2 * DUAL64_BYTES, "the exchange area must fit the K buffers");
    float* xch = reinterpret_cast<float*>(lds_all) + wave * (CT * 16 * 64) + lane;
    if (kl == 1) {
#pragma unroll
      for (int t = 0; t < CT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) xch[(16 * t + r) * 64] = cx.dq[t][r];
    }
    __syncthreads();
    if (kl == 1) return;
#pragma unroll
    for (int t = 0; t < CT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) cx.dq[t][r] += xch[(16 * t + r) * 64];
  }
  if (q_ok) store_acc_t<CT>(dQ + ((int64_t)head * d.nq + q_row) * H, cx.dq, cx.half, d.scale, H, g.acc != 0);
}

}  // namespace

bool bwd_mfma_supported(const a2d_tile_desc& d) {
  return d.dtype == A2D_BF16 && (d.hdim == 128 || d.hdim == 96 || d.hdim == 80 || d.hdim == 64);
}

// Bytes of the dS workspace of a tile (0 when the hand-over does not apply: a sub-block that does
// not start at a multiple of 64 keys, or 4 GiB or more per key/value head)
size_t bwd_ds_bytes(const a2d_tile_desc& d, const SegList& g) {
  if (!bwd_mfma_supported(d)) return 0;
  for (int s = 0; s < g.n; ++s)
    if (g.start[s] % 64 != 0) return 0;
  const size_t per_head = ds_head_bytes(d.nq, d.nkv);
  if (per_head * (size_t)g.group >= ((size_t)1 << 32)) return 0;   // 32-bit offsets inside a key/value head's share
  return per_head * (size_t)d.heads;
}

namespace {
template <int HR>
hipError_t bwd_launch_ds(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                         const void* V, const void* dO, const float* lse, const float* delta, float* dQ, float* dK,
                         float* dV, void* ds_ws, hipStream_t s) {
  constexpr int DSQ_LDS = 2 * DUAL64_BYTES;
  const bool grouped = g.group > 1;
  int cus = 0;
  hipError_t e = device_cus(&cus);
  if (e != hipSuccess) return e;
  const bool big = (int64_t)d.heads * ((d.nq + 255) / 256) >= cus;
  // the dQ kernel walks the keys in two lanes when at most one 128-row block comes to a compute unit
  const bool lanes = !big && (int64_t)d.heads * ((d.nq + 127) / 128) <= cus;
  if (ph == PREPARE) {
    e = ensure_dynamic_lds(grouped ? reinterpret_cast<const void*>(bwd_dkdv_kernel<HR, true, true>)
                                   : reinterpret_cast<const void*>(bwd_dkdv_kernel<HR, false, true>), DK_LDS);
    if (e != hipSuccess) return e;
    return lanes ? ensure_dynamic_lds(reinterpret_cast<const void*>(bwd_dq_ds_kernel<8, HR, 2>), 2 * DSQ_LDS)
                 : ensure_dynamic_lds(big ? reinterpret_cast<const void*>(bwd_dq_ds_kernel<8, HR, 1>)
                                          : reinterpret_cast<const void*>(bwd_dq_ds_kernel<4, HR, 1>), DSQ_LDS);
  }
  dim3 grid_kv(xcd_grid(d.heads / g.group * g.qsplit, (d.nkv + DK_KEYS - 1) / DK_KEYS));
  const int dq_rows = big ? 256 : 128;
  const int per_unit = g.group / g.split;
  dim3 grid_q(xcd_grid(d.heads / per_unit, per_unit * ((d.nq + dq_rows - 1) / dq_rows)));
  if (grouped)
    A2D_LAUNCH((bwd_dkdv_kernel<HR, true, true>), grid_kv, dim3(DK_THREADS), DK_LDS, s, d, g,
                       (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dK, dV,
                       (bf16_t*)ds_ws);
  else
    A2D_LAUNCH((bwd_dkdv_kernel<HR, false, true>), grid_kv, dim3(DK_THREADS), DK_LDS, s, d, g,
                       (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dK, dV,
                       (bf16_t*)ds_ws);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (big)
    A2D_LAUNCH((bwd_dq_ds_kernel<8, HR, 1>), grid_q, dim3(512), DSQ_LDS, s, d, g, (const bf16_t*)K,
                       (const bf16_t*)ds_ws, dQ);
  else if (lanes)
    A2D_LAUNCH((bwd_dq_ds_kernel<8, HR, 2>), grid_q, dim3(512), 2 * DSQ_LDS, s, d, g, (const bf16_t*)K,
                       (const bf16_t*)ds_ws, dQ);
  else
    A2D_LAUNCH((bwd_dq_ds_kernel<4, HR, 1>), grid_q, dim3(256), DSQ_LDS, s, d, g, (const bf16_t*)K,
                       (const bf16_t*)ds_ws, dQ);
  return hipGetLastError();
}

template <int HR>
hipError_t bwd_launch_hd(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                         const void* V, const void* dO, const float* lse, const float* delta, float* dQ, float* dK,
                         float* dV, void* ds_ws, hipStream_t s) {
  if (ds_ws) return bwd_launch_ds<HR>(ph, d, g, Q, K, V, dO, lse, delta, dQ, dK, dV, ds_ws, s);
  constexpr int DQ_LDS = dq_lds(padded_head(HR));
  const bool grouped = g.group > 1;
  // Q and dO in the plain layout: the variant with compile-time staging offsets
  const bool plain = d.lq.row == HR && d.ldo.row == HR && d.lq.head == (int64_t)d.nq * HR && d.ldo.head == d.lq.head;
  // dQ kernel: 256-row workgroups unless that leaves compute units without a workgroup
  int cus = 0;
  hipError_t e = device_cus(&cus);
  if (e != hipSuccess) return e;
  const bool big = (int64_t)d.heads * ((d.nq + 255) / 256) >= cus;
  // two key lanes when at most one 128-row block comes to a compute unit
  const bool lanes = !big && (int64_t)d.heads * ((d.nq + 127) / 128) <= cus;
  if (ph == PREPARE) {
    const void* dkdv = plain ? (grouped ? reinterpret_cast<const void*>(bwd_dkdv_kernel<HR, true, false, true>)
                                        : reinterpret_cast<const void*>(bwd_dkdv_kernel<HR, false, false, true>))
                             : (grouped ? reinterpret_cast<const void*>(bwd_dkdv_kernel<HR, true, false, false>)
                                        : reinterpret_cast<const void*>(bwd_dkdv_kernel<HR, false, false, false>));
    e = ensure_dynamic_lds(dkdv, DK_LDS);
    if (e != hipSuccess) return e;
    return lanes ? ensure_dynamic_lds(reinterpret_cast<const void*>(bwd_dq_kernel<8, HR, 2>), 2 * DQ_LDS)
                 : ensure_dynamic_lds(big ? reinterpret_cast<const void*>(bwd_dq_kernel<8, HR, 1>)
                                          : reinterpret_cast<const void*>(bwd_dq_kernel<4, HR, 1>), DQ_LDS);
  }
  dim3 grid_kv(xcd_grid(d.heads / g.group * g.qsplit, (d.nkv + DK_KEYS - 1) / DK_KEYS));
  const int dq_rows = big ? 256 : 128;
  const int per_unit = g.group / g.split;
  dim3 grid_q(xcd_grid(d.heads / per_unit, per_unit * ((d.nq + dq_rows - 1) / dq_rows)));
#define A2D_DKDV(GR, PL)                                                                                          \
  A2D_LAUNCH((bwd_dkdv_kernel<HR, GR, false, PL>), grid_kv, dim3(DK_THREADS), DK_LDS, s, d, g, (const bf16_t*)Q, \
                     (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dK, dV, (bf16_t*)nullptr)
  if (grouped && plain) A2D_DKDV(true, true);
  else if (grouped) A2D_DKDV(true, false);
  else if (plain) A2D_DKDV(false, true);
  else A2D_DKDV(false, false);
#undef A2D_DKDV
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (big)
    A2D_LAUNCH((bwd_dq_kernel<8, HR, 1>), grid_q, dim3(512), DQ_LDS, s, d, g, (const bf16_t*)Q,
                       (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dQ);
  else if (lanes)
    A2D_LAUNCH((bwd_dq_kernel<8, HR, 2>), grid_q, dim3(512), 2 * DQ_LDS, s, d, g, (const bf16_t*)Q,
                       (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dQ);
  else
    A2D_LAUNCH((bwd_dq_kernel<4, HR, 1>), grid_q, dim3(256), DQ_LDS, s, d, g, (const bf16_t*)Q,
                       (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, delta, dQ);
  return hipGetLastError();
}
}  // namespace

// How many workgroups should share a key block of a grouped-head dK/dV launch (each walking
// group / Z of the query heads): the divisor Z of `group` (at most A2D_MAX_PARTS) that minimises
// rounds of workgroups over the compute units x query heads per workgroup; the smallest on a tie.
int choose_qsplit(int kv_heads, int group, int key_blocks, int cus) {
  int best = 1;
  int64_t best_cost = -1;
  for (int z = 1; z <= group && z <= A2D_MAX_PARTS; ++z) {
    if (group % z != 0) continue;
    const int64_t wgs = (int64_t)kv_heads * z * key_blocks;
    const int64_t cost = ((wgs + cus - 1) / cus) * (group / z);
    if (best_cost < 0 || cost < best_cost) { best = z; best_cost = cost; }
  }
  return best;
}

// ds_ws != NULL: a workspace of bwd_ds_bytes(d, g) bytes; the dK/dV kernel leaves dS there and the
// dQ kernel is the contraction-only one.
// split_ws != NULL (grouped heads): room for 2 * min(group, A2D_MAX_PARTS) partial buffers of
// [key/value heads][nkv][H] floats; the query heads of a group may then be split over several
// workgroups per key block (choose_qsplit) whose dK / dV sums a sum kernel adds up.
hipError_t launch_bwd_mfma(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                           const void* V, const void* dO, const float* lse, const float* delta, float* dQ,
                           float* dK, float* dV, void* ds_ws, float* split_ws, hipStream_t s) {
  SegList gg = g;
  gg.qsplit = 1;
  float* dKo = dK;
  float* dVo = dV;
  const int kv_heads = d.heads / g.group;
  const int64_t n = (int64_t)kv_heads * d.nkv * d.hdim;        // elements of dK (of dV)
  if (split_ws && g.group > 1) {
    int cus = 0;
    const hipError_t e = device_cus(&cus);
    if (e != hipSuccess) return e;
    gg.qsplit = choose_qsplit(kv_heads, g.group, (d.nkv + DK_KEYS - 1) / DK_KEYS, cus);
    if (gg.qsplit > 1) {
      dKo = split_ws;
      dVo = split_ws + (int64_t)gg.qsplit * n;
    }
  }
  hipError_t e;
  if (d.hdim == 128) e = bwd_launch_hd<128>(ph, d, gg, Q, K, V, dO, lse, delta, dQ, dKo, dVo, ds_ws, s);
  else if (d.hdim == 96) e = bwd_launch_hd<96>(ph, d, gg, Q, K, V, dO, lse, delta, dQ, dKo, dVo, ds_ws, s);
  else if (d.hdim == 80) e = bwd_launch_hd<80>(ph, d, gg, Q, K, V, dO, lse, delta, dQ, dKo, dVo, ds_ws, s);
  else e = bwd_launch_hd<64>(ph, d, gg, Q, K, V, dO, lse, delta, dQ, dKo, dVo, ds_ws, s);
  if (e != hipSuccess || gg.qsplit == 1 || ph == PREPARE) return e;   // (the sum kernel needs no preparation)
  // dK = sum_z partial z (in order of z: bitwise reproducible), the same for dV
  SumPtrs pk, pv;
  for (int z = 0; z < A2D_MAX_PARTS; ++z) { pk.p[z] = nullptr; pv.p[z] = nullptr; }
  for (int z = 0; z < gg.qsplit; ++z) { pk.p[z] = dKo + (int64_t)z * n; pv.p[z] = dVo + (int64_t)z * n; }
  e = launch_fix_bwd(gg.qsplit, n, d.hdim / 4, A2D_F32, pk, plain_out(), dK, s);
  if (e != hipSuccess) return e;
  return launch_fix_bwd(gg.qsplit, n, d.hdim / 4, A2D_F32, pv, plain_out(), dV, s);
}

}  // namespace a2d
