// bf16 MFMA forward tile kernel for H = 128, 96, 80 and 64 (Sec. 3.1, Eq. (3), evaluated block by
// block with the recurrence of Sec. 2.2).
//
// Work split: one workgroup = 8 wavefronts = 256 query rows of one head; each
// wavefront owns 32 query rows for the whole kernel and walks the key blocks
// (64 keys per step) that the workgroup stages through LDS.  (Tiles with too few
// query blocks for that take 128-row workgroups: see the kernel's template parameters.)
//
// Both contractions are issued TRANSPOSED so that no cross-lane data movement is
// needed between them (v_mfma_f32_32x32x16_bf16, D = A * B, A: 32 x 16, B: 16 x 32):
//   S^T = K * Q^T : A = K fragment (LDS, 128-bit reads), B = Q^T fragment (registers,
//                   loaded once).  In D a lane holds 16 keys of ONE query column, so
//                   row max / row sum are in-lane reductions; the two lanes of a row
//                   (lane, lane ^ 32) are combined only when needed.
//   O^T += V^T * P^T : B = P^T is exactly the D layout of S^T (the contraction index
//                   may be permuted freely as long as A uses the same permutation),
//                   A = V^T fragment read from the row-major V tile with the LDS
//                   transpose read ds_read_b64_tr_b16.
// LDS: K and V tiles double-buffered, rows padded (K: 272 B, V: 320 B) so that the
// 128-bit K reads and the transposing V reads are bank-conflict free and every
// fragment address is one per-lane base register plus an immediate.  One workgroup
// fills a compute unit with two wavefronts per SIMD, so one's MFMAs overlap the other's
// softmax arithmetic, and every staged K / V tile serves all eight (two workgroups of four
// would stage each tile twice: measured 6 % slower).
//
// Rescaling is lazy: a row's exponent reference m_ref follows its running maximum
// only when a score exceeds it by more than 2^8 (in the exponent's units) - a rare,
// wave-uniform branch, and the only place where the two lanes of a row talk to each
// other.  Each lane tracks the true maximum of its own scores; at the end the halves
// are combined and N, l are brought to the true row maximum, so (N, m, l) leave the
// kernel exactly as Eq. (3) defines them.
#include "a2d_mfma.hpp"

namespace a2d {
namespace {

using namespace mfma;

constexpr int BN = 64;             // keys per step
constexpr int VLD = 320;           // V tile row stride, bytes (256 of data at most + a pad that shifts rows by 16 banks)
// K tile row stride: the row's bytes + 16, which shifts consecutive rows by one 128-bit bank group
__host__ __device__ constexpr int kld(int hd) { return hd * 2 + 16; }
__host__ __device__ constexpr int buf_bytes(int hd) { return BN * kld(hd) + BN * VLD; }
__host__ __device__ constexpr int lds_bytes(int hd) { return 2 * buf_bytes(hd); }
constexpr float kRescaleThreshold = 8.0f;   // log2 units

template <int HD>
struct FwdState {
  f32x16 o[HD / 32];
  float m_lane;   // true running max of this lane's raw dot products
  float m_ref;    // reference the exponentials are taken against (raw units, same in both lanes of a row)
  float l_run;    // this lane's share of the row sum, relative to m_ref
};

// One 64-key block for one wavefront.  k_rd / v_rd: per-lane LDS byte addresses of the
// natural K fragment (t = 0, st = 0) and of the transposing V read (u = 0, ht = 0, low rows).
// KS slices of H in the score contraction (those that hold data: a head size of 80 fills five of
// the padded six), HD / 32 column tiles in the output contraction.
template <int HD, bool MASK, int KS = HD / 16>
__device__ __forceinline__ void fwd_block(FwdState<HD>& st, const bf16x8 (&qf)[HD / 16], unsigned k_rd, unsigned v_rd,
                                          int k0, int my_vis, int half, float c) {
  constexpr int CT = HD / 32, KLD = kld(HD);
  // K fragments go through a ring four deep: each is requested four MFMAs before its use (the
  // scheduling fences keep the compiler from sinking the requests back to their uses)
  f32x16 s[2];
  s[0] = zero16();
  s[1] = zero16();
  bf16x8 kr[4];
  // step I works on key tile I & 1, slice I >> 1 of H: the two accumulators alternate, so that no
  // MFMA accumulates onto the result of the one issued just before it
  auto ldk = [&](auto I) {
    constexpr int i = decltype(I)::value;
    kr[i & 3] = lds_load_b128(k_rd + (i & 1) * 32 * KLD + (i >> 1) * 32);
  };
  static_for<0, 4>(ldk);
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, 2 * KS>([&](auto I) {
    constexpr int i = decltype(I)::value;
    s[i & 1] = mma(kr[i & 3], qf[i >> 1], s[i & 1]);
    if constexpr (i + 4 < 2 * KS) ldk(std::integral_constant<int, i + 4>{});
    __builtin_amdgcn_sched_barrier(0);
  });
  if (MASK) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = k0 + 32 * t + 8 * (r >> 2) + 4 * half + (r & 3);
        if (key >= my_vis) s[t][r] = -INFINITY;
      }
  }
  float mx = s[0][0];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
  st.m_lane = fmaxf(st.m_lane, mx);
  // (m_lane - m_ref) is +inf on the first visible block, NaN (-> false) while nothing is visible
  const bool grow = (st.m_lane - st.m_ref) * c > kRescaleThreshold;
  if (__builtin_amdgcn_ballot_w64(grow) != 0) {
    asm volatile("" ::: "memory");   // keep this a real (rarely taken) branch: no if-conversion
    const float m_row = fmaxf(st.m_lane, __shfl_xor(st.m_lane, 32, 64));
    const float m_use = (m_row == -INFINITY) ? 0.f : m_row;
    const float alpha = fast_exp2((st.m_ref - m_use) * c);    // m_ref = -inf gives 0
    st.m_ref = m_row;
    st.l_run *= alpha;
#pragma unroll
    for (int t = 0; t < CT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[t][r] *= alpha;
  }
  const float mc = (st.m_ref == -INFINITY) ? 0.f : st.m_ref * c;
  // V^T fragments (step I: 16-key group I / CT, column tile I % CT) go through a ring four deep
  // as well; the first four are requested before the exponentials
  bf16x8 vr[4];
  auto ldv = [&](auto I) {
    constexpr int i = decltype(I)::value;
    const unsigned a = v_rd + (i / CT) * 16 * VLD + (i % CT) * 64;
    vr[i & 3] = lds_load_tr(a, a + 8 * VLD);
  };
  static_for<0, 4>(ldv);
  __builtin_amdgcn_sched_barrier(0);
  float psum = 0.f;
  bf16x8 pb[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float p = fast_exp2(fmaf(s[u >> 1][8 * (u & 1) + e], c, -mc));
      psum += p;
      pb[u][e] = (bf16_t)p;
    }
  st.l_run += psum;
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, 4 * CT>([&](auto I) {
    constexpr int i = decltype(I)::value;
    st.o[i % CT] = mma(vr[i & 3], pb[i / CT], st.o[i % CT]);
    if constexpr (i + 4 < 4 * CT) ldv(std::integral_constant<int, i + 4>{});
    __builtin_amdgcn_sched_barrier(0);
  });
}

// WAVES wavefronts per workgroup, in KL key lanes of WAVES / KL wavefronts (32 query rows each):
//   <8, 1>  256 rows: one workgroup fills a compute unit;
//   <4, 1>  128 rows, two workgroups per compute unit: when there are too few 256-row blocks to
//           give every compute unit one;
//   <8, 2>  128 rows walked by two key lanes: when even the 128-row blocks come to at most one per
//           compute unit, so that a SIMD still holds two wavefronts.  The lanes take alternate key
//           blocks of the walk, each staging its own tiles into its own pair of LDS buffers, and
//           their (N, m, l) are merged through LDS at the end exactly as two partials of one
//           query block are (Alg. 2).
// HR: head size = row length in memory (80, 96 or 128); the LDS tiles and fragments are laid out
// for the padded head size HD = padded_head(HR) (96 or 128).
template <int WAVES, int HR, int KL>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void fwd_mfma_kernel(
    a2d_tile_desc d, SegList g, const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, float* __restrict__ O_part, float* __restrict__ m_out,
    float* __restrict__ l_out) {
  constexpr int RW = WAVES / KL;          // wavefronts of one key lane
  constexpr int BM = 32 * RW;             // query rows per workgroup
  constexpr int kThreads = 64 * RW;       // threads of one key lane (they stage its tiles)
  constexpr int HD = padded_head(HR), H = HR;
  constexpr int KS = HD / 16, CT = HD / 32, KLD = kld(HD), K_BYTES = BN * KLD, BUF_BYTES = buf_bytes(HD);
  constexpr int KSR = (HR + 15) / 16;     // slices of H that hold data
  constexpr int kLdsBytes = lds_bytes(HD);
  extern __shared__ __attribute__((aligned(16))) char lds_all[];
  // per key lane: [buf]{ K tile (BN x KLD), V tile (BN x VLD) }
  const int kl = KL == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / kThreads);   // key lane of this wavefront
  char* const lds = lds_all + kl * kLdsBytes;
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

  const int nqb = (d.nq + BM - 1) / BM;
  // the query blocks of the query heads that share a key/value head go to one XCD (to g.split
  // XCDs, an equal share of the heads each, when that is what spreads the load evenly)
  int unit, blk;
  const int per_unit = g.group / g.split;
  if (!xcd_map(d.heads / per_unit, per_unit * nqb, g.by_size != 0, unit, blk)) return;
  // (blocks numbered by size first when the workgroups are ordered by size)
  const int head = unit * per_unit + (g.by_size ? blk % per_unit : blk / nqb), kvh = head / g.group;
  blk = g.by_size ? blk / per_unit : blk % nqb;
  // heavy (late) query blocks first: under a causal mask they walk more key blocks
  const int q0 = (nqb - 1 - blk) * BM;
  const int tid = (int)threadIdx.x - kl * kThreads;     // within the key lane
  const int wave = tid >> 6, lane = tid & 63;
  const int half = lane >> 5, l32 = lane & 31;
  Q += (int64_t)head * d.lq.head;
  K += (int64_t)kvh * d.lk.head;
  V += (int64_t)kvh * d.lv.head;

  // ---- Q^T fragments: lane holds query row (l32), h = 16*step + 8*half + 0..7.
  // Rows beyond nq re-read the last row (their results are never stored).
  const int q_row = q0 + wave * 32 + l32;
  bf16x8 qf[KS];
  {
    const bf16_t* qp = Q + (int64_t)min(q_row, d.nq - 1) * d.lq.row + 8 * half;
#pragma unroll
    for (int x = 0; x < KS; ++x) {
      if (16 * x < H) qf[x] = *reinterpret_cast<const bf16x8*>(qp + 16 * x);
      else qf[x] = bf16x8{};                                  // columns past the head size are zero
    }
  }
  FwdState<HD> st;
#pragma unroll
  for (int t = 0; t < CT; ++t) st.o[t] = zero16();
  st.l_run = 0.f;
  const float c = d.scale * kLog2e;
  float m_in = -INFINITY;
  if (g.acc) {
    // (key lane 0 continues the stored partial; the barriers are the whole workgroup's)
    // Continue from the (N, m, l) already in the output buffers: N into the accumulators (same
    // element mapping as the epilogue's stores), m as the exponent reference, l into one of the two
    // lanes of the row.  A lane's share of N is 16 scattered 16-byte pieces of its row, so the
    // rows come in through LDS: each wavefront reads 16 of its rows at a time with whole-row
    // coalesced loads into a private, padded LDS area and the owning lanes pick their pieces.
    constexpr int ALD = HD * 4 + 16;                          // padded row stride, bytes
    static_assert(16 * ALD * (kThreads / 64) <= kLdsBytes, "accumulator staging must fit the tile buffers");
    char* area = lds_all + wave * 16 * ALD;
    const int64_t wrow0 = (int64_t)head * d.nq + q0 + wave * 32;   // first row of the wavefront
    const int64_t last_row = (int64_t)head * d.nq + d.nq - 1;
    const bool col_ok = 4 * (lane & 31) < H;                 // this lane's 16-byte piece exists in the row
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      u32x4 t[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {                          // two whole rows per load instruction
        const int64_t r = wrow0 + 16 * pass + 2 * i + (lane >> 5);
        t[i] = u32x4{0, 0, 0, 0};
        if (col_ok && kl == 0)
          t[i] = *reinterpret_cast<const u32x4*>(O_part + (r < last_row ? r : last_row) * H + 4 * (lane & 31));
      }
      if (4 * (lane & 31) < HD && kl == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          *reinterpret_cast<u32x4*>(area + (2 * i + (lane >> 5)) * ALD + 16 * (lane & 31)) = t[i];
      }
      __syncthreads();
      if ((l32 >> 4) == pass && kl == 0) {
        const char* mine = area + (l32 & 15) * ALD + 16 * half;
#pragma unroll
        for (int ht = 0; ht < CT; ++ht)
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(mine + (32 * ht + 8 * gq) * 4);
            st.o[ht][4 * gq] = v[0]; st.o[ht][4 * gq + 1] = v[1]; st.o[ht][4 * gq + 2] = v[2]; st.o[ht][4 * gq + 3] = v[3];
          }
      }
      __syncthreads();
    }
    if (kl != 0) {
      // the other key lane starts from nothing
    } else if (q_row < d.nq) {
      const int64_t row = (int64_t)head * d.nq + q_row;
      m_in = m_out[row];
      st.l_run = half == 0 ? l_out[row] : 0.f;
    } else {
#pragma unroll
      for (int t = 0; t < CT; ++t) st.o[t] = zero16();       // rows beyond nq: nothing to continue
    }
  }
  wait_vmem_all();
  st.m_lane = st.m_ref = m_in / d.scale;               // -inf stays -inf

  // ---- visibility, per key/value sub-block s: query i sees the first vis_count(i, s) keys of it
  // (key kk of the sub-block iff kk <= i + rel[s])
  auto vis_count = [&](int i, int s) -> int {
    if (!d.causal) return g.rows[s];
    const int64_t v = (int64_t)i + g.rel[s] + 1;
    return v <= 0 ? 0 : (v < g.rows[s] ? (int)v : g.rows[s]);
  };
  const int blk_last = min(q0 + BM, d.nq) - 1;
  const int w_first = min(q0 + wave * 32, d.nq - 1);
  const int w_last = min(q0 + wave * 32 + 31, d.nq - 1);
  // key blocks of sub-block s that some row of the workgroup sees; the walk over (sub-block, block)
  auto seg_blocks = [&](int s) { return (vis_count(blk_last, s) + BN - 1) / BN; };
  int nvis_wave = 0, nfull_wave = 0, my_vis = 0;   // of the current sub-block
  auto enter_segment = [&](int s) {
    nvis_wave = vis_count(w_last, s);        // keys any row of the wave sees
    nfull_wave = vis_count(w_first, s);      // keys every row of the wave sees
    my_vis = vis_count(min(q_row, d.nq - 1), s);
  };


  // ---- staging: thread moves the 16-byte chunk (tid & 15) of rows (tid >> 4) + 32 p.
  // Rows beyond nkv re-read the last row: finite values, masked out of the scores.
  const int ld_row = tid >> 4, ld_chunk = tid & 15;
  const bool ld_ok = ld_chunk * 8 < H;          // the chunk exists in memory (else it is a zero pad column group)
  const bool st_ok = ld_chunk * 8 < HD;         // the chunk exists in the LDS tile
  const int k_wr = ld_row * KLD + ld_chunk * 16;
  const int v_wr = K_BYTES + ld_row * VLD + ld_chunk * 16;
  constexpr int ST_ROWS = kThreads / 16, ST_N = BN / ST_ROWS;   // rows per pass, passes per tile
  u32x4 kreg[ST_N], vreg[ST_N];
#pragma unroll
  for (int p = 0; p < ST_N; ++p) { kreg[p] = u32x4{0, 0, 0, 0}; vreg[p] = u32x4{0, 0, 0, 0}; }
  // block j of the sub-block of seg_rows keys that starts at local key seg_start; rows beyond its
  // end re-read its last row
  // (row strides in bytes, pinned in registers: read from the kernel arguments inside the loop they
  // would be scalar loads, which share a wait counter with the LDS reads in flight.  A head's rows
  // span less than 4 GiB - the API layer checks it - so row index times stride fits 32 bits.)
  const unsigned k_row_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.lk.row * 2);
  const unsigned v_row_bytes = __builtin_amdgcn_readfirstlane((unsigned)d.lv.row * 2);
  auto load_tile = [&](int seg_start, int seg_rows, int j) {
    const int k0 = seg_start + j * BN;
    const gptr_t kb = uniform_gptr(reinterpret_cast<const char*>(K) + (unsigned)k0 * k_row_bytes);   // scalar bases
    const gptr_t vb = uniform_gptr(reinterpret_cast<const char*>(V) + (unsigned)k0 * v_row_bytes);
    const int last = seg_rows - 1 - j * BN;
    if (ld_ok) {
#pragma unroll
      for (int p = 0; p < ST_N; ++p) {
        const unsigned r = (unsigned)min(ld_row + ST_ROWS * p, last);
        kreg[p] = gload_b128(kb, __umul24(r, k_row_bytes) + ld_chunk * 16);
        vreg[p] = gload_b128(vb, __umul24(r, v_row_bytes) + ld_chunk * 16);
      }
    }
  };
  auto store_tile = [&](int boff) {
    if (st_ok) {
#pragma unroll
      for (int p = 0; p < ST_N; ++p) {
        *reinterpret_cast<u32x4*>(lds + boff + k_wr + p * ST_ROWS * KLD) = kreg[p];
        *reinterpret_cast<u32x4*>(lds + boff + v_wr + p * ST_ROWS * VLD) = vreg[p];
      }
    }
  };
  // fragment read bases (buffer 0)
  const unsigned k_rd0 = lds_base + l32 * KLD + half * 16;
  const int g16 = lane >> 4, j16 = lane & 15;
  const unsigned v_rd0 =
      lds_base + K_BYTES + (4 * (g16 >> 1) + (j16 >> 2)) * VLD + (16 * (g16 & 1) + 4 * (j16 & 3)) * 2;

  // Walk over the entries (sub-block, key block); key lane kl takes entries kl, kl + KL, ...  The
  // sub-block table lives in kernel-argument memory, and scalar loads share a wait counter with the
  // LDS reads in flight, so it is only touched when a walk moves to another sub-block; in between
  // its values sit in registers.
  // An entry is (sub-block sb, block j of its nblk); sb == g.n: past the end.
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
    load_tile(nx_start, nx_rows, j);
    store_tile(0);
  }
  __syncthreads();

  int boff = 0;
  while ((KL == 1 ? sb : lead_sb) < g.n) {
    int nsb = sb, nj = j, nnblk = nblk;
#pragma unroll
    for (int x = 0; x < KL; ++x) advance(nsb, nj, nnblk);
    const bool more = nsb < g.n;
    if (more && nsb != sb) { nx_start = g.start[nsb]; nx_rows = g.rows[nsb]; }
    if (more) load_tile(nx_start, nx_rows, nj);
    const int k0 = j * BN;                         // local to the sub-block
    if ((KL == 1 || sb < g.n) && k0 < nvis_wave) {
      if (k0 + BN > nfull_wave) fwd_block<HD, true, KSR>(st, qf, k_rd0 + boff, v_rd0 + boff, k0, my_vis, half, c);
      else fwd_block<HD, false, KSR>(st, qf, k_rd0 + boff, v_rd0 + boff, k0, my_vis, half, c);
    }
    if (more) store_tile(BUF_BYTES - boff);
    __syncthreads();
    if (more && nsb != sb) enter_segment(nsb);
    if (KL > 1) {
#pragma unroll
      for (int x = 0; x < KL; ++x) advance(lead_sb, lead_j, lead_nblk);
    }
    sb = nsb; j = nj; nblk = nnblk;
    boff = BUF_BYTES - boff;
  }

  // ---- epilogue: bring N and l to the true row maximum, store N, m (scaled units), l
  float m_row = fmaxf(st.m_lane, __shfl_xor(st.m_lane, 32, 64));
  float f = (m_row == -INFINITY) ? 0.f : fast_exp2((st.m_ref - m_row) * c);
  float l_tot = (st.l_run + __shfl_xor(st.l_run, 32, 64)) * f;
  if constexpr (KL == 2) {
    // Key lane 1 hands its (N, m, l) to lane 0 through LDS (the tiles are no longer read: every
    // wavefront has passed the walk's last barrier), which merges the two as Alg. 2 does.
    // Layout: [row wavefront][value index][lane], one float each, so every access is conflict free.
    constexpr int NV = CT * 16 + 2;
    static_assert(RW * NV * 256 <= KL * kLdsBytes, "the exchange area must fit the tile buffers");
    float* xch = reinterpret_cast<float*>(lds_all) + wave * NV * 64 + lane;
    if (kl == 1) {
#pragma unroll
      for (int t = 0; t < CT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) xch[(16 * t + r) * 64] = st.o[t][r] * f;
      xch[(CT * 16) * 64] = m_row;
      xch[(CT * 16 + 1) * 64] = l_tot;
    }
    __syncthreads();
    if (kl == 1) return;
    const float m1 = xch[(CT * 16) * 64], l1 = xch[(CT * 16 + 1) * 64];
    const float m_new = fmaxf(m_row, m1);
    const float a0 = (m_row == -INFINITY) ? 0.f : f * fast_exp2((m_row - m_new) * c);
    const float a1 = (m1 == -INFINITY) ? 0.f : fast_exp2((m1 - m_new) * c);
#pragma unroll
    for (int t = 0; t < CT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[t][r] = st.o[t][r] * a0 + xch[(16 * t + r) * 64] * a1;
    l_tot = (m_row == -INFINITY ? 0.f : l_tot * fast_exp2((m_row - m_new) * c)) + l1 * a1;
    m_row = m_new;
    f = 1.f;
  }
  // a lane's piece (column tile ht, group gq) covers columns 32 ht + 8 gq + 4 half + 0..3
  if (q_row < d.nq && g.norm) {
    // normalised partial: O' = N / l rounded to bf16, lse' = m + ln l (Sec. 3.2, footnote)
    const int64_t row = (int64_t)head * d.nq + q_row;
    const float fn = l_tot > 0.f ? f / l_tot : 0.f;
    bf16_t* op = reinterpret_cast<bf16_t*>(O_part) + row * H + 4 * half;
#pragma unroll
    for (int ht = 0; ht < CT; ++ht)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 v;
        v[0] = (bf16_t)(st.o[ht][4 * gq] * fn); v[1] = (bf16_t)(st.o[ht][4 * gq + 1] * fn);
        v[2] = (bf16_t)(st.o[ht][4 * gq + 2] * fn); v[3] = (bf16_t)(st.o[ht][4 * gq + 3] * fn);
        if (32 * ht + 8 * gq + 4 * half < H) *reinterpret_cast<bf16x4*>(op + 32 * ht + 8 * gq) = v;
      }
    if (half == 0) m_out[row] = l_tot > 0.f ? m_row * d.scale + logf(l_tot) : -INFINITY;
  } else if (q_row < d.nq) {
    const int64_t row = (int64_t)head * d.nq + q_row;
    float* op = O_part + row * H + 4 * half;
#pragma unroll
    for (int ht = 0; ht < CT; ++ht)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        f32x4 v = {st.o[ht][4 * gq] * f, st.o[ht][4 * gq + 1] * f, st.o[ht][4 * gq + 2] * f,
                   st.o[ht][4 * gq + 3] * f};
        if (32 * ht + 8 * gq + 4 * half < H) *reinterpret_cast<f32x4*>(op + 32 * ht + 8 * gq) = v;
      }
    if (half == 0) {
      m_out[row] = m_row * d.scale;      // -inf stays -inf (scale > 0)
      l_out[row] = l_tot;
    }
  }
}

}  // namespace

bool fwd_mfma_supported(const a2d_tile_desc& d) {
  return d.dtype == A2D_BF16 && (d.hdim == 128 || d.hdim == 96 || d.hdim == 80 || d.hdim == 64);
}

namespace {
template <int WAVES, int HR, int KL>
hipError_t fwd_launch(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K, const void* V,
                      float* O_part, float* m, float* l, hipStream_t s) {
  constexpr int bytes = KL * lds_bytes(padded_head(HR)), BM = 32 * WAVES / KL;
  if (ph == PREPARE)
    return ensure_dynamic_lds(reinterpret_cast<const void*>(fwd_mfma_kernel<WAVES, HR, KL>), bytes);
  const int per_unit = g.group / g.split;
  dim3 grid(xcd_grid(d.heads / per_unit, per_unit * ((d.nq + BM - 1) / BM))), block(64 * WAVES);
  A2D_LAUNCH((fwd_mfma_kernel<WAVES, HR, KL>), grid, block, bytes, s, d, g, (const bf16_t*)Q,
                     (const bf16_t*)K, (const bf16_t*)V, O_part, m, l);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_fwd_mfma(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                           const void* V, float* O_part, float* m, float* l, hipStream_t s) {
  // 256-row workgroups unless that leaves compute units without one; then 128-row workgroups, with
  // two key lanes when at most one of those comes to a compute unit either
  int cus = 0;
  const hipError_t e = device_cus(&cus);
  if (e != hipSuccess) return e;
  const bool big = (int64_t)d.heads * ((d.nq + 255) / 256) >= cus;
  const bool lanes = !big && (int64_t)d.heads * ((d.nq + 127) / 128) <= cus;
#define A2D_FWD(HR)                                                                      \
  return big     ? fwd_launch<8, HR, 1>(ph, d, g, Q, K, V, O_part, m, l, s)              \
         : lanes ? fwd_launch<8, HR, 2>(ph, d, g, Q, K, V, O_part, m, l, s)              \
                 : fwd_launch<4, HR, 1>(ph, d, g, Q, K, V, O_part, m, l, s)
  if (d.hdim == 128) { A2D_FWD(128); }
  if (d.hdim == 96) { A2D_FWD(96); }
  if (d.hdim == 80) { A2D_FWD(80); }
  A2D_FWD(64);
#undef A2D_FWD
}

}  // namespace a2d
