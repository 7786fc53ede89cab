// Shared device-side helpers and the launcher interface between the C-ABI layer
// (a2d_api.hip) and the kernel translation units.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "a2d.h"

namespace a2d {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }

// 2^x and log2(x) on the hardware transcendental unit (about 1 ulp).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

template <typename T> struct dtype_of;
template <> struct dtype_of<float> { static constexpr int value = A2D_F32; };
template <> struct dtype_of<bf16_t> { static constexpr int value = A2D_BF16; };

// Key/value sub-blocks of a tile for the causal mask.  Sub-block s covers the local keys
// start[s] .. start[s] + rows[s] - 1 (the sub-blocks tile 0 .. nkv - 1 in order) and its keys are
// consecutive tokens; rel[s] = q_off - (global index of its first key).  Query row i (local) sees
// key start[s] + kk of sub-block s iff kk <= i + rel[s].  A plain tile is one sub-block.
// `acc` rides along: != 0 makes the forward start from the (N, m, l) already in its output
// buffers and the backward add to the dQ partial already in its output buffer.
// `norm` != 0: the forward writes the NORMALISED partial O' = N / l in the input dtype (into the
// buffer passed as O_part) and lse' = m + ln l (into the buffer passed as m) instead of (N, m, l).
// `group` >= 1: query heads per key/value head (grouped-query attention: query head h reads
// key/value head h / group; K, V, dK, dV have heads / group heads).  `split` divides `group`:
// kernels that own query blocks place the query heads of a key/value head on XCDs in `split`
// separate runs (1 = all of them on one XCD; chosen by group_split()).
// `by_size` != 0: the blocks of the tile differ in cost (a causal mask crosses it); the kernels then
// order their workgroups by block, heaviest first, over a whole XCD (see xcd_map).
struct SegList {
  int n;
  int acc;
  int norm;
  int group;
  int split;
  int by_size;
  int qsplit;     // dK/dV kernel, grouped heads: workgroups per key block, each walking group / qsplit query heads
  int start[A2D_MAX_SEGMENTS];
  int rows[A2D_MAX_SEGMENTS];
  int64_t rel[A2D_MAX_SEGMENTS];
};

// Smallest divisor s of `group` that makes kv_heads * s a multiple of the 8 XCDs (an even load per
// XCD); `group` itself (one run per query head) when there is none.
inline int group_split(int kv_heads, int group) {
  for (int s = 1; s <= group; ++s)
    if (group % s == 0 && (kv_heads * s) % 8 == 0) return s;
  return group;
}

// sub-block that holds local key c (c < nkv)
__device__ __forceinline__ int seg_of_key(const SegList& g, int c) {
  int s = 0;
  while (s + 1 < g.n && c >= g.start[s + 1]) ++s;
  return s;
}
// does query row i see local key c (causal mask)?
__device__ __forceinline__ bool seg_visible(const SegList& g, int i, int c) {
  const int s = seg_of_key(g, c);
  return (int64_t)(c - g.start[s]) <= (int64_t)i + g.rel[s];
}

// ---- per-process caches of HIP runtime queries (a2d_device.hip; thread-safe) ----
// compute units of the current device
hipError_t device_cus(int* cus);
// raises the kernel's dynamic-LDS limit to `bytes` once per (device, kernel)
hipError_t ensure_dynamic_lds(const void* kernel, int bytes);
// Debugging aid: route every tile call to the vector-ALU kernels.  The default comes from
// A2D_FORCE_GENERIC=1 in the environment, read once per process; a2d_debug_force_generic() sets it.
bool force_generic();
void set_force_generic(bool on);
// Kernel trace of the calling host thread (diagnostic, see a2d_debug_trace): trace_mark records
// the next caller-supplied event on the stream; a no-op (one thread-local test) when no trace is set.
void trace_set(hipEvent_t* events, int n);
int trace_count();
void trace_mark(hipStream_t s);
// every kernel launch of the method goes through this: the launch, then the trace mark
#define A2D_LAUNCH(kernel, grid, block, lds, stream, ...)               \
  do {                                                                  \
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);  \
    ::a2d::trace_mark(stream);                                          \
  } while (0)

// ---- launchers (none synchronises) ----
// Every tile launcher runs in two phases so that a call can finish everything that may fail on the
// host side before its first kernel is enqueued: PREPARE only raises the dynamic-LDS limits of the
// kernels the LAUNCH phase of the same arguments will use (cached per device), LAUNCH only
// launches and returns the launch's hipError_t.
enum Phase { PREPARE = 0, LAUNCH = 1 };

// Generic tile kernels: fp32 arithmetic on the vector ALUs for fp32 or bf16
// inputs, any nq / nkv, H in {64, 80, 96, 128}.
hipError_t launch_fwd_generic(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                              const void* V, float* O_part, float* m, float* l, hipStream_t s);
hipError_t launch_bwd_generic(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                              const void* V, const void* dO, const float* lse, const float* delta, float* dQ,
                              float* dK, float* dV, hipStream_t s);

// delta[head][row] = sum_j dO[head][row][j] * O[head][row][j]  (O, dO with the layouts d.lo, d.ldo)
hipError_t launch_delta(const a2d_tile_desc& d, const void* O, const void* dO, float* delta, hipStream_t s);

// bf16 MFMA tile kernels (H in {64, 80, 96, 128}).  `supported` tells whether the shape is covered.
bool fwd_mfma_supported(const a2d_tile_desc& d);
hipError_t launch_fwd_mfma(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                           const void* V, float* O_part, float* m, float* l, hipStream_t s);
bool bwd_mfma_supported(const a2d_tile_desc& d);
// ds_ws: NULL, or a workspace of bwd_ds_bytes(d, g) (> 0) bytes through which the dK/dV kernel
// hands dS to a contraction-only dQ kernel (instead of the dQ kernel recomputing S and dP)
size_t bwd_ds_bytes(const a2d_tile_desc& d, const SegList& g);
hipError_t launch_bwd_mfma(Phase ph, const a2d_tile_desc& d, const SegList& g, const void* Q, const void* K,
                           const void* V, const void* dO, const float* lse, const float* delta, float* dQ,
                           float* dK, float* dV, void* ds_ws, float* split_ws, hipStream_t s);
// the dK/dV kernel's choice of workgroups per key block for grouped heads (see launch_bwd_mfma)
int choose_qsplit(int kv_heads, int group, int key_blocks, int cus);

struct FixPtrs {
  const float* o[A2D_MAX_PARTS];
  const float* m[A2D_MAX_PARTS];
  const float* l[A2D_MAX_PARTS];
};
struct SumPtrs {
  const float* p[A2D_MAX_PARTS];
};
// Layout of a merge's output in the model's dtype: plain != 0 -> [rows][H] contiguous; else row r of
// head h (nq rows per head) starts h * head + r * row elements from the base.
struct OutMap {
  int64_t head;
  int64_t row;
  int nq;
  int plain;
};
inline OutMap plain_out() { return OutMap{0, 0, 1, 1}; }
hipError_t launch_fix(int k, int64_t rows, int hdim, int out_dtype, const FixPtrs& p, const OutMap& om, void* O,
                      float* lse, hipStream_t s);
hipError_t launch_attnfix(int k, int64_t rows, int hdim, const FixPtrs& p, float* N, float* m, float* l,
                          hipStream_t s);
// (hv = 4-column groups per row, used only when the output is not plain)
hipError_t launch_fix_bwd(int k, int64_t n, int hv, int out_dtype, const SumPtrs& p, const OutMap& om, void* out,
                          hipStream_t s);
// merge of k NORMALISED partials (O'_k in in_dtype, lse_k)
struct NormPtrs {
  const void* o[A2D_MAX_PARTS];
  const float* lse[A2D_MAX_PARTS];
};
hipError_t launch_fix_norm(int k, int64_t rows, int hdim, int in_dtype, int out_dtype, const NormPtrs& p,
                           const OutMap& om, void* O, float* lse, hipStream_t s);

// plain device copy of n16 16-byte pieces (diagnostic: HBM ceiling and counter calibration)
hipError_t launch_copy_probe(void* dst, const void* src, size_t n16, hipStream_t s);
// MFMA-only ceiling probe (diagnostic)
hipError_t launch_mfma_probe(int blocks, int iters, int random_data, float* scratch, hipStream_t s);
// model of the forward loop: MFMA + one LDS fragment per MFMA + softmax arithmetic (diagnostic)
hipError_t launch_mix_probe(int blocks, int iters, float* scratch, hipStream_t s);
hipError_t launch_bwd_mix_probe(int blocks, int iters, int leave_out, float* scratch, hipStream_t s);
hipError_t launch_lds_read_probe(int blocks, int iters, int kind, float* scratch, hipStream_t s);
int mfma_probe_threads();
int mfma_probe_mfma_per_iter();

}  // namespace a2d
