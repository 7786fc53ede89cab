// C-ABI layer of liba2d: argument validation, kernel selection, error reporting.
// No arithmetic happens here; see include/a2d.h for the contract of every call.
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "a2d_common.hpp"

namespace {

thread_local char g_err[512] = "";

a2d_status fail(a2d_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

#define A2D_TRY(expr)                   \
  do {                                  \
    a2d_status st__ = (expr);           \
    if (st__ != A2D_OK) return st__;    \
  } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

a2d_status check_desc(const a2d_tile_desc* d, const char* who) {
  if (!d) return fail(A2D_ERR_INVALID_ARG, "%s: descriptor is NULL", who);
  if (d->heads < 1 || d->nq < 1 || d->nkv < 1)
    return fail(A2D_ERR_INVALID_ARG, "%s: heads=%d nq=%d nkv=%d must all be >= 1", who, d->heads,
                d->nq, d->nkv);
  if (d->dtype != A2D_F32 && d->dtype != A2D_BF16)
    return fail(A2D_ERR_UNSUPPORTED, "%s: dtype %d is neither A2D_F32 nor A2D_BF16", who, d->dtype);
  if (d->hdim != 64 && d->hdim != 80 && d->hdim != 96 && d->hdim != 128)
    return fail(A2D_ERR_UNSUPPORTED, "%s: head size %d not supported (64, 80, 96 or 128)", who, d->hdim);
  if (!(d->scale > 0.f) || !std::isfinite(d->scale))
    return fail(A2D_ERR_INVALID_ARG, "%s: scale must be finite and > 0", who);
  if (d->causal != 0 && d->causal != 1)
    return fail(A2D_ERR_INVALID_ARG, "%s: causal must be 0 or 1", who);
  if (d->heads > 65535) return fail(A2D_ERR_INVALID_ARG, "%s: heads=%d exceeds 65535", who, d->heads);
  if (d->nq > (1 << 22) || d->nkv > (1 << 22))   // the kernels address a head's rows with 32-bit byte offsets
    return fail(A2D_ERR_INVALID_ARG, "%s: nq=%d / nkv=%d exceed 2^22 rows", who, d->nq, d->nkv);
  const int64_t lim = (int64_t)1 << 40;
  if (d->q_off < -lim || d->q_off > lim || d->kv_off < -lim || d->kv_off > lim)
    return fail(A2D_ERR_INVALID_ARG, "%s: offsets out of range", who);
  if ((d->flags & ~A2D_DESC_KEEP_DS) != 0)
    return fail(A2D_ERR_INVALID_ARG, "%s: desc->flags=%d: only A2D_DESC_KEEP_DS is defined", who, d->flags);
  return A2D_OK;
}

// One layout of the descriptor: {0, 0} becomes the plain one; anything else is checked.  `heads`
// consecutive heads of `rows` rows are addressed through one base pointer with 32-bit byte offsets.
a2d_status resolve_layout(a2d_layout* l, const char* name, int64_t heads, int64_t rows, const a2d_tile_desc* d,
                          const char* who) {
  const int64_t esize = d->dtype == A2D_BF16 ? 2 : 4, unit = 16 / esize;
  if (l->head == 0 && l->row == 0) {
    l->row = d->hdim;
    l->head = rows * d->hdim;
    return A2D_OK;
  }
  if (l->row < d->hdim || l->head < 1 || l->row > ((int64_t)1 << 40) || l->head > ((int64_t)1 << 40))
    return fail(A2D_ERR_INVALID_ARG, "%s: layout of %s: head=%lld row=%lld (row >= H and head >= 1 needed)", who,
                name, (long long)l->head, (long long)l->row);
  if (l->row % unit != 0 || l->head % unit != 0)
    return fail(A2D_ERR_MISALIGNED, "%s: layout of %s: head=%lld row=%lld must be multiples of %lld elements", who,
                name, (long long)l->head, (long long)l->row, (long long)unit);
  // (the kernels form row offsets with 24-bit multiplies: rows < 2^22, row stride < 16 MiB)
  if (l->row * esize >= ((int64_t)1 << 24))
    return fail(A2D_ERR_UNSUPPORTED, "%s: layout of %s: row stride of %lld bytes (16 MiB or more)", who, name,
                (long long)(l->row * esize));
  const int64_t span = ((heads - 1) * l->head + (rows - 1) * l->row + d->hdim) * esize;
  if (span >= ((int64_t)1 << 32))
    return fail(A2D_ERR_UNSUPPORTED, "%s: layout of %s: %lld head(s) of %lld rows span %lld bytes (4 GiB or more)",
                who, name, (long long)heads, (long long)rows, (long long)span);
  return A2D_OK;
}

// The descriptor with every layout the call uses filled in (group = query heads per key/value head)
a2d_status resolve_layouts(const a2d_tile_desc* desc, int group, bool backward, const char* who, a2d_tile_desc* out) {
  *out = *desc;
  A2D_TRY(resolve_layout(&out->lq, "Q", group, desc->nq, desc, who));
  A2D_TRY(resolve_layout(&out->lk, "K", 1, desc->nkv, desc, who));
  A2D_TRY(resolve_layout(&out->lv, "V", 1, desc->nkv, desc, who));
  if (backward) {
    A2D_TRY(resolve_layout(&out->lo, "O", group, desc->nq, desc, who));
    A2D_TRY(resolve_layout(&out->ldo, "dO", group, desc->nq, desc, who));
  }
  return A2D_OK;
}

a2d_status check_ptr(const void* p, const char* who, const char* name) {
  if (!p) return fail(A2D_ERR_INVALID_ARG, "%s: %s is NULL", who, name);
  if (!aligned16(p)) return fail(A2D_ERR_MISALIGNED, "%s: %s is not 16-byte aligned", who, name);
  return A2D_OK;
}

a2d_status hip_result(hipError_t e, const char* who) {
  if (e == hipSuccess) return A2D_OK;
  return fail(A2D_ERR_HIP, "%s: HIP error %d (%s)", who, (int)e, hipGetErrorString(e));
}

// the plain tile as one sub-block
a2d::SegList one_segment(const a2d_tile_desc* d) {
  a2d::SegList g;
  memset(&g, 0, sizeof(g));
  g.n = 1;
  g.group = 1;
  g.split = 1;
  g.qsplit = 1;
  g.start[0] = 0;
  g.rows[0] = d->nkv;
  g.rel[0] = d->q_off - d->kv_off;
  return g;
}

a2d_status make_segments(const a2d_tile_desc* d, int nseg, const a2d_kv_segment* segs, const char* who,
                         a2d::SegList* g) {
  if (nseg < 1 || nseg > A2D_MAX_SEGMENTS)
    return fail(A2D_ERR_INVALID_ARG, "%s: nseg=%d outside 1..%d", who, nseg, A2D_MAX_SEGMENTS);
  if (!segs) return fail(A2D_ERR_INVALID_ARG, "%s: segs is NULL", who);
  memset(g, 0, sizeof(*g));
  g->n = nseg;
  g->group = 1;
  g->split = 1;
  g->qsplit = 1;
  int64_t total = 0;
  for (int s = 0; s < nseg; ++s) {
    if (segs[s].rows < 1 || segs[s].pad != 0)
      return fail(A2D_ERR_INVALID_ARG, "%s: segs[%d]: rows=%d must be >= 1 and pad 0", who, s, segs[s].rows);
    if (segs[s].kv_off < -((int64_t)1 << 60) || segs[s].kv_off > ((int64_t)1 << 60))
      return fail(A2D_ERR_INVALID_ARG, "%s: segs[%d].kv_off out of range", who, s);
    g->start[s] = (int)total;
    g->rows[s] = segs[s].rows;
    g->rel[s] = d->q_off - segs[s].kv_off;
    total += segs[s].rows;
    if (total > d->nkv) break;
  }
  if (total != d->nkv)
    return fail(A2D_ERR_INVALID_ARG, "%s: the sub-blocks hold %lld keys, desc->nkv is %d", who,
                (long long)total, d->nkv);
  return A2D_OK;
}

// Do the blocks of the tile differ much in cost?  Under a causal mask the last query row may see
// many more keys than the first (at least twice as many: a tile the diagonal crosses); the kernels
// then start their workgroups heaviest first over a whole XCD instead of head by head.  (A
// gathered key row whose last sub-block alone is cut by the diagonal stays head by head: its
// blocks cost nearly the same and the heads' rows are worth more in L2.)
int blocks_differ(const a2d_tile_desc* d, const a2d::SegList& g) {
  if (!d->causal) return 0;
  auto vis = [&](int64_t i, int s) -> int64_t {
    const int64_t v = i + g.rel[s] + 1;
    return v <= 0 ? 0 : (v < g.rows[s] ? v : g.rows[s]);
  };
  int64_t first = 0, last = 0;
  for (int s = 0; s < g.n; ++s) { first += vis(0, s); last += vis(d->nq - 1, s); }
  return last >= 2 * first && last > first;
}

a2d_status partial_fwd_impl(const a2d_tile_desc* desc, const a2d::SegList& g, const void* Q, const void* K,
                            const void* V, float* O_part, float* m, float* l, void* stream,
                            const char* who) {
  A2D_TRY(check_ptr(Q, who, "Q"));
  A2D_TRY(check_ptr(K, who, "K"));
  A2D_TRY(check_ptr(V, who, "V"));
  A2D_TRY(check_ptr(O_part, who, "O_part"));
  A2D_TRY(check_ptr(m, who, "m"));
  A2D_TRY(check_ptr(l, who, "l"));
  hipStream_t s = static_cast<hipStream_t>(stream);
  a2d_tile_desc dd;
  A2D_TRY(resolve_layouts(desc, g.group, false, who, &dd));
  if (!a2d::force_generic() && a2d::fwd_mfma_supported(dd)) {
    a2d::SegList go = g;
    go.by_size = blocks_differ(desc, g);
    A2D_TRY(hip_result(a2d::launch_fwd_mfma(a2d::PREPARE, dd, go, Q, K, V, O_part, m, l, s), who));
    a2d::trace_mark(s);
    return hip_result(a2d::launch_fwd_mfma(a2d::LAUNCH, dd, go, Q, K, V, O_part, m, l, s), who);
  }
  A2D_TRY(hip_result(a2d::launch_fwd_generic(a2d::PREPARE, dd, g, Q, K, V, O_part, m, l, s), who));
  a2d::trace_mark(s);
  return hip_result(a2d::launch_fwd_generic(a2d::LAUNCH, dd, g, Q, K, V, O_part, m, l, s), who);
}

a2d_status partial_bwd_impl(const a2d_tile_desc* desc, const a2d::SegList& g, const void* Q, const void* K,
                            const void* V, const void* O, const void* dO, const float* lse,
                            float* dQ_part, float* dK_part, float* dV_part, void* workspace,
                            size_t workspace_bytes, void* stream, const char* who, bool split_groups = false) {
  A2D_TRY(check_ptr(Q, who, "Q"));
  A2D_TRY(check_ptr(K, who, "K"));
  A2D_TRY(check_ptr(V, who, "V"));
  A2D_TRY(check_ptr(O, who, "O"));
  A2D_TRY(check_ptr(dO, who, "dO"));
  A2D_TRY(check_ptr(lse, who, "lse"));
  A2D_TRY(check_ptr(dQ_part, who, "dQ_part"));
  A2D_TRY(check_ptr(dK_part, who, "dK_part"));
  A2D_TRY(check_ptr(dV_part, who, "dV_part"));
  const bool keep_ds = (desc->flags & A2D_DESC_KEEP_DS) != 0;
  const size_t delta_bytes = a2d_workspace_bytes(desc, A2D_OP_PARTIAL_BWD, 0);
  const size_t need = keep_ds ? a2d_workspace_bytes(desc, A2D_OP_PARTIAL_BWD_DS, 0) : delta_bytes;
  // a value no allocation can have (a foreign caller that passed a 32-bit integer for the size_t,
  // leaving the upper half undefined) is refused
  if (workspace_bytes > ((size_t)1 << 46))
    return fail(A2D_ERR_INVALID_ARG, "%s: workspace_bytes = %zu is not a plausible size (size_t expected)", who,
                workspace_bytes);
  if (!workspace || workspace_bytes < need)
    return fail(A2D_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need,
                workspace ? workspace_bytes : (size_t)0);
  if (!aligned16(workspace)) return fail(A2D_ERR_MISALIGNED, "%s: workspace is not 16-byte aligned", who);
  hipStream_t s = static_cast<hipStream_t>(stream);
  a2d_tile_desc dd;
  A2D_TRY(resolve_layouts(desc, g.group, true, who, &dd));
  // the partial dK / dV buffers of a split over the group's query heads lie behind the dS area
  float* split_ws = nullptr;
  if (split_groups && g.group > 1) {
    const size_t all = a2d_workspace_bytes(desc, A2D_OP_PARTIAL_BWD_SPLIT, desc->heads / g.group);
    if (workspace_bytes < all)
      return fail(A2D_ERR_WORKSPACE, "%s: A2D_TILE_SPLIT_GROUPS needs a workspace of %zu bytes, %zu given", who, all,
                  workspace_bytes);
    split_ws = reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                        a2d_workspace_bytes(desc, A2D_OP_PARTIAL_BWD_DS, 0));
  }
  float* delta = static_cast<float*>(workspace);
  if (!a2d::force_generic() && a2d::bwd_mfma_supported(dd)) {
    // the dS hand-over when the caller asked for it and this tile allows it (`need` covers the
    // plain tile's dS area; a gathered tile of the same nkv has the same size or none)
    const size_t ds_bytes = keep_ds ? a2d::bwd_ds_bytes(dd, g) : 0;
    void* ds_ws = (ds_bytes > 0 && workspace_bytes >= delta_bytes + ds_bytes) ? static_cast<char*>(workspace) + delta_bytes
                                                                              : nullptr;
    a2d::SegList go = g;
    go.by_size = blocks_differ(desc, g);
    A2D_TRY(hip_result(a2d::launch_bwd_mfma(a2d::PREPARE, dd, go, Q, K, V, dO, lse, delta, dQ_part, dK_part,
                                            dV_part, ds_ws, split_ws, s), who));
    a2d::trace_mark(s);
    A2D_TRY(hip_result(a2d::launch_delta(dd, O, dO, delta, s), who));
    return hip_result(a2d::launch_bwd_mfma(a2d::LAUNCH, dd, go, Q, K, V, dO, lse, delta, dQ_part, dK_part,
                                           dV_part, ds_ws, split_ws, s), who);
  }
  A2D_TRY(hip_result(a2d::launch_bwd_generic(a2d::PREPARE, dd, g, Q, K, V, dO, lse, delta, dQ_part, dK_part,
                                             dV_part, s), who));
  a2d::trace_mark(s);
  A2D_TRY(hip_result(a2d::launch_delta(dd, O, dO, delta, s), who));
  return hip_result(a2d::launch_bwd_generic(a2d::LAUNCH, dd, g, Q, K, V, dO, lse, delta, dQ_part, dK_part,
                                            dV_part, s), who);
}

// ---- scratch of the entry point that allocates nothing (a2d_partial_bwd_static): the per-row
// sums delta of one backward call, at most A2D_STATIC_MAX_ROWS of them, in a file-scope device
// array.  Every GPU the library runs on holds its own copy at its own address until the process
// ends; host code only ever uses the address hipGetSymbolAddress returned for the current device.
__device__ __align__(256) float scratch[A2D_STATIC_MAX_ROWS];
constexpr int kMaxDevices = 64;
std::atomic<float*> g_scratch_ptr[kMaxDevices];

a2d_status static_scratch(float** out, const char* who) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_result(e, who);
  if (dev < 0 || dev >= kMaxDevices)
    return fail(A2D_ERR_UNSUPPORTED, "%s: device index %d outside 0..%d", who, dev, kMaxDevices - 1);
  float* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {                                     // first call on this device (it is the current one)
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_result(e, who);
    if (!sym) return fail(A2D_ERR_HIP, "%s: hipGetSymbolAddress returned NULL", who);
    p = static_cast<float*>(sym);
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // (two first calls at once store the same address)
  }
  *out = p;
  return A2D_OK;
}

}  // namespace

extern "C" {

a2d_status a2d_partial_bwd_static(const a2d_tile_desc* desc, const void* Q, const void* K, const void* V,
                                  const void* O, const void* dO, const float* lse, float* dQ_part,
                                  float* dK_part, float* dV_part, void* stream) {
  const char* who = "a2d_partial_bwd_static";
  A2D_TRY(check_desc(desc, who));
  if ((desc->flags & A2D_DESC_KEEP_DS) != 0)
    return fail(A2D_ERR_UNSUPPORTED, "%s: A2D_DESC_KEEP_DS needs a caller workspace (use a2d_partial_bwd)", who);
  const int64_t rows = (int64_t)desc->heads * desc->nq;
  if (rows > (int64_t)A2D_STATIC_MAX_ROWS)
    return fail(A2D_ERR_WORKSPACE, "%s: heads * nq = %lld rows exceed the static scratch of %d rows (use a2d_partial_bwd)",
                who, (long long)rows, A2D_STATIC_MAX_ROWS);
  float* ptr = nullptr;
  A2D_TRY(static_scratch(&ptr, who));
  // delta is written in full by the call's first kernel before the others read it: nothing in
  // the array has to start at zero
  return partial_bwd_impl(desc, one_segment(desc), Q, K, V, O, dO, lse, dQ_part, dK_part, dV_part, ptr,
                          sizeof(float) * (size_t)A2D_STATIC_MAX_ROWS, stream, who);
}

size_t a2d_workspace_bytes(const a2d_tile_desc* desc, int op, int k) {
  if (!desc || desc->heads < 1 || desc->nq < 1) return 0;
  if (op != A2D_OP_PARTIAL_BWD && op != A2D_OP_PARTIAL_BWD_DS && op != A2D_OP_PARTIAL_BWD_SPLIT) return 0;
  const size_t rows = (size_t)desc->heads * (size_t)desc->nq;
  const size_t delta_bytes = ((rows * sizeof(float) + 255) / 256) * 256;
  if (op == A2D_OP_PARTIAL_BWD || desc->nkv < 1) return delta_bytes;
  // (the dS area is sized for the plain tile whether or not a call ends up using it, so that the
  // areas behind it have a fixed place)
  const size_t ds_area = ((a2d::bwd_ds_bytes(*desc, one_segment(desc)) + 255) / 256) * 256;
  if (op == A2D_OP_PARTIAL_BWD_DS) return delta_bytes + ds_area;
  // partial dK / dV of a split over the group's query heads: 2 x min(group, A2D_MAX_PARTS) buffers
  const int kv_heads = (k >= 1 && desc->heads % k == 0) ? k : desc->heads;
  const int group = desc->heads / kv_heads;
  const size_t parts = group < A2D_MAX_PARTS ? group : A2D_MAX_PARTS;
  return delta_bytes + ds_area + 2 * parts * (size_t)kv_heads * desc->nkv * desc->hdim * sizeof(float);
}

a2d_status a2d_partial_fwd_seg(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, float* O_part,
                               float* m, float* l, void* /*workspace*/, size_t /*workspace_bytes*/,
                               void* stream) {
  const char* who = "a2d_partial_fwd_seg";
  A2D_TRY(check_desc(desc, who));
  a2d::SegList g;
  A2D_TRY(make_segments(desc, nseg, segs, who, &g));
  return partial_fwd_impl(desc, g, Q, K, V, O_part, m, l, stream, who);
}

a2d_status a2d_partial_fwd_norm(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                                const void* Q, const void* K, const void* V, void* O_norm,
                                float* lse_part, void* /*workspace*/, size_t /*workspace_bytes*/,
                                void* stream) {
  const char* who = "a2d_partial_fwd_norm";
  A2D_TRY(check_desc(desc, who));
  a2d::SegList g = one_segment(desc);
  if (nseg != 0) A2D_TRY(make_segments(desc, nseg, segs, who, &g));
  g.norm = 1;
  // the kernels take the normalised output through the O_part argument and lse' through m; l is unused
  return partial_fwd_impl(desc, g, Q, K, V, static_cast<float*>(O_norm), lse_part, lse_part, stream, who);
}

}  // extern "C"

namespace {
a2d_status out_map(const a2d_layout* lo, int64_t nq, int32_t hdim, int32_t out_dtype, const char* who, a2d::OutMap* om);

a2d_status fix_norm_impl(int k, int64_t rows, int32_t hdim, int32_t in_dtype, int32_t out_dtype,
                         const void* const* O_norm_parts, const float* const* lse_parts, void* O,
                         const a2d::OutMap& om, float* lse, void* stream, const char* who) {
  if (k < 1 || k > A2D_MAX_PARTS)
    return fail(A2D_ERR_INVALID_ARG, "%s: k=%d outside 1..%d", who, k, A2D_MAX_PARTS);
  if (rows < 1) return fail(A2D_ERR_INVALID_ARG, "%s: rows=%lld must be >= 1", who, (long long)rows);
  if (hdim < 4 || hdim % 4 != 0 || hdim > 1024)
    return fail(A2D_ERR_UNSUPPORTED, "%s: hdim=%d must be a multiple of 4 in 4..1024", who, hdim);
  if ((in_dtype != A2D_F32 && in_dtype != A2D_BF16) || (out_dtype != A2D_F32 && out_dtype != A2D_BF16))
    return fail(A2D_ERR_UNSUPPORTED, "%s: dtype %d / %d not supported", who, in_dtype, out_dtype);
  if (rows * (int64_t)(hdim / 4) > ((int64_t)1 << 39))
    return fail(A2D_ERR_INVALID_ARG, "%s: rows * hdim too large", who);
  if (!O_norm_parts || !lse_parts) return fail(A2D_ERR_INVALID_ARG, "%s: pointer array is NULL", who);
  A2D_TRY(check_ptr(O, who, "O"));
  A2D_TRY(check_ptr(lse, who, "lse"));
  a2d::NormPtrs p;
  memset(&p, 0, sizeof(p));
  for (int x = 0; x < k; ++x) {
    A2D_TRY(check_ptr(O_norm_parts[x], who, "O_norm_parts[x]"));
    A2D_TRY(check_ptr(lse_parts[x], who, "lse_parts[x]"));
    p.o[x] = O_norm_parts[x]; p.lse[x] = lse_parts[x];
  }
  a2d::trace_mark(static_cast<hipStream_t>(stream));
  return hip_result(a2d::launch_fix_norm(k, rows, hdim, in_dtype, out_dtype, p, om, O, lse,
                                         static_cast<hipStream_t>(stream)), who);
}
}  // namespace

extern "C" {

a2d_status a2d_fix_norm(int k, int64_t rows, int32_t hdim, int32_t in_dtype, int32_t out_dtype,
                        const void* const* O_norm_parts, const float* const* lse_parts, void* O,
                        float* lse, void* stream) {
  return fix_norm_impl(k, rows, hdim, in_dtype, out_dtype, O_norm_parts, lse_parts, O, a2d::plain_out(), lse,
                       stream, "a2d_fix_norm");
}

a2d_status a2d_fix_norm_strided(int k, int32_t heads, int32_t nq, int32_t hdim, int32_t in_dtype,
                                int32_t out_dtype, const void* const* O_norm_parts,
                                const float* const* lse_parts, void* O, const a2d_layout* lo, float* lse,
                                void* stream) {
  const char* who = "a2d_fix_norm_strided";
  if (heads < 1 || nq < 1) return fail(A2D_ERR_INVALID_ARG, "%s: heads=%d nq=%d must be >= 1", who, heads, nq);
  a2d::OutMap om;
  A2D_TRY(out_map(lo, nq, hdim, out_dtype, who, &om));
  return fix_norm_impl(k, (int64_t)heads * nq, hdim, in_dtype, out_dtype, O_norm_parts, lse_parts, O, om, lse,
                       stream, who);
}

// query heads per key/value head, or an error
static a2d_status group_of(const a2d_tile_desc* desc, int kv_heads, const char* who, a2d::SegList* g) {
  int* group = &g->group;
  if (kv_heads < 1 || desc->heads % kv_heads != 0)
    return fail(A2D_ERR_INVALID_ARG, "%s: kv_heads=%d must be >= 1 and divide heads=%d", who, kv_heads,
                desc->heads);
  *group = desc->heads / kv_heads;
  if ((int64_t)*group * desc->nq > ((int64_t)1 << 22))
    return fail(A2D_ERR_INVALID_ARG, "%s: group * nq = %lld exceeds 2^22 rows", who,
                (long long)*group * desc->nq);
  g->split = a2d::group_split(kv_heads, *group);
  return A2D_OK;
}

a2d_status a2d_partial_fwd_gqa(const a2d_tile_desc* desc, int32_t kv_heads, int nseg,
                               const a2d_kv_segment* segs, int flags, const void* Q, const void* K,
                               const void* V, void* out0, float* out1, float* out2,
                               void* /*workspace*/, size_t /*workspace_bytes*/, void* stream) {
  const char* who = "a2d_partial_fwd_gqa";
  A2D_TRY(check_desc(desc, who));
  if (flags != 0 && flags != A2D_TILE_ACCUMULATE && flags != A2D_TILE_NORMALISED)
    return fail(A2D_ERR_INVALID_ARG, "%s: flags=%d must be 0, A2D_TILE_ACCUMULATE or A2D_TILE_NORMALISED", who, flags);
  a2d::SegList g = one_segment(desc);
  if (nseg != 0) A2D_TRY(make_segments(desc, nseg, segs, who, &g));
  A2D_TRY(group_of(desc, kv_heads, who, &g));
  g.acc = flags == A2D_TILE_ACCUMULATE;
  g.norm = flags == A2D_TILE_NORMALISED;
  return partial_fwd_impl(desc, g, Q, K, V, static_cast<float*>(out0), out1, g.norm ? out1 : out2, stream, who);
}

a2d_status a2d_partial_bwd_gqa(const a2d_tile_desc* desc, int32_t kv_heads, int nseg,
                               const a2d_kv_segment* segs, int flags, const void* Q, const void* K,
                               const void* V, const void* O, const void* dO, const float* lse,
                               float* dQ_part, float* dK_part, float* dV_part, void* workspace,
                               size_t workspace_bytes, void* stream) {
  const char* who = "a2d_partial_bwd_gqa";
  A2D_TRY(check_desc(desc, who));
  if ((flags & ~(A2D_TILE_ACCUMULATE | A2D_TILE_SPLIT_GROUPS)) != 0)
    return fail(A2D_ERR_INVALID_ARG, "%s: flags=%d: only A2D_TILE_ACCUMULATE and A2D_TILE_SPLIT_GROUPS apply", who, flags);
  a2d::SegList g = one_segment(desc);
  if (nseg != 0) A2D_TRY(make_segments(desc, nseg, segs, who, &g));
  A2D_TRY(group_of(desc, kv_heads, who, &g));
  g.acc = (flags & A2D_TILE_ACCUMULATE) != 0;
  return partial_bwd_impl(desc, g, Q, K, V, O, dO, lse, dQ_part, dK_part, dV_part, workspace,
                          workspace_bytes, stream, who, (flags & A2D_TILE_SPLIT_GROUPS) != 0);
}

a2d_status a2d_partial_fwd_acc(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, float* O_part,
                               float* m, float* l, void* /*workspace*/, size_t /*workspace_bytes*/,
                               void* stream) {
  const char* who = "a2d_partial_fwd_acc";
  A2D_TRY(check_desc(desc, who));
  a2d::SegList g = one_segment(desc);
  if (nseg != 0) A2D_TRY(make_segments(desc, nseg, segs, who, &g));
  g.acc = 1;
  return partial_fwd_impl(desc, g, Q, K, V, O_part, m, l, stream, who);
}

a2d_status a2d_partial_fwd(const a2d_tile_desc* desc, const void* Q, const void* K, const void* V,
                           float* O_part, float* m, float* l, void* /*workspace*/,
                           size_t /*workspace_bytes*/, void* stream) {
  const char* who = "a2d_partial_fwd";
  A2D_TRY(check_desc(desc, who));
  return partial_fwd_impl(desc, one_segment(desc), Q, K, V, O_part, m, l, stream, who);
}

}  // extern "C"

namespace {

// layout of a merge's output: NULL or {0, 0} = plain
a2d_status out_map(const a2d_layout* lo, int64_t nq, int32_t hdim, int32_t out_dtype, const char* who, a2d::OutMap* om) {
  *om = a2d::plain_out();
  if (!lo || (lo->head == 0 && lo->row == 0)) return A2D_OK;
  const int64_t unit = out_dtype == A2D_BF16 ? 8 : 4;
  if (lo->row < hdim || lo->head < 1 || lo->row > ((int64_t)1 << 40) || lo->head > ((int64_t)1 << 40))
    return fail(A2D_ERR_INVALID_ARG, "%s: output layout: head=%lld row=%lld (row >= H and head >= 1 needed)", who,
                (long long)lo->head, (long long)lo->row);
  if (lo->row % unit != 0 || lo->head % unit != 0)
    return fail(A2D_ERR_MISALIGNED, "%s: output layout: head=%lld row=%lld must be multiples of %lld elements", who,
                (long long)lo->head, (long long)lo->row, (long long)unit);
  om->head = lo->head; om->row = lo->row; om->nq = (int)nq; om->plain = 0;
  return A2D_OK;
}

a2d_status fix_impl(int k, int64_t rows, int32_t hdim, int32_t out_dtype,
                    const float* const* O_parts, const float* const* m, const float* const* l,
                    void* O, const a2d::OutMap& om, float* lse, void* stream, const char* who) {
  if (k < 1 || k > A2D_MAX_PARTS)
    return fail(A2D_ERR_INVALID_ARG, "%s: k=%d outside 1..%d", who, k, A2D_MAX_PARTS);
  if (rows < 1) return fail(A2D_ERR_INVALID_ARG, "%s: rows=%lld must be >= 1", who, (long long)rows);
  if (hdim < 4 || hdim % 4 != 0 || hdim > 1024)
    return fail(A2D_ERR_UNSUPPORTED, "%s: hdim=%d must be a multiple of 4 in 4..1024", who, hdim);
  if (out_dtype != A2D_F32 && out_dtype != A2D_BF16)
    return fail(A2D_ERR_UNSUPPORTED, "%s: out_dtype %d not supported", who, out_dtype);
  if (rows * (int64_t)(hdim / 4) > ((int64_t)1 << 39))
    return fail(A2D_ERR_INVALID_ARG, "%s: rows * hdim too large", who);
  if (!O_parts || !m || !l) return fail(A2D_ERR_INVALID_ARG, "%s: pointer array is NULL", who);
  A2D_TRY(check_ptr(O, who, "O"));
  A2D_TRY(check_ptr(lse, who, "lse"));
  a2d::FixPtrs p;
  memset(&p, 0, sizeof(p));
  for (int x = 0; x < k; ++x) {
    A2D_TRY(check_ptr(O_parts[x], who, "O_parts[x]"));
    A2D_TRY(check_ptr(m[x], who, "m[x]"));
    A2D_TRY(check_ptr(l[x], who, "l[x]"));
    p.o[x] = O_parts[x]; p.m[x] = m[x]; p.l[x] = l[x];
  }
  a2d::trace_mark(static_cast<hipStream_t>(stream));
  return hip_result(a2d::launch_fix(k, rows, hdim, out_dtype, p, om, O, lse,
                                    static_cast<hipStream_t>(stream)), who);
}

a2d_status fix_bwd_impl(int k, int64_t n, int32_t hdim, int32_t out_dtype, const float* const* parts, void* out,
                        const a2d::OutMap& om, void* stream, const char* who) {
  if (k < 1 || k > A2D_MAX_PARTS)
    return fail(A2D_ERR_INVALID_ARG, "%s: k=%d outside 1..%d", who, k, A2D_MAX_PARTS);
  if (n < 4 || n % 4 != 0)
    return fail(A2D_ERR_INVALID_ARG, "%s: n=%lld must be a positive multiple of 4", who, (long long)n);
  if (n > ((int64_t)1 << 41)) return fail(A2D_ERR_INVALID_ARG, "%s: n too large", who);
  if (out_dtype != A2D_F32 && out_dtype != A2D_BF16)
    return fail(A2D_ERR_UNSUPPORTED, "%s: out_dtype %d not supported", who, out_dtype);
  if (!parts) return fail(A2D_ERR_INVALID_ARG, "%s: parts is NULL", who);
  A2D_TRY(check_ptr(out, who, "out"));
  a2d::SumPtrs p;
  memset(&p, 0, sizeof(p));
  for (int x = 0; x < k; ++x) {
    A2D_TRY(check_ptr(parts[x], who, "parts[x]"));
    p.p[x] = parts[x];
  }
  a2d::trace_mark(static_cast<hipStream_t>(stream));
  return hip_result(a2d::launch_fix_bwd(k, n, hdim / 4, out_dtype, p, om, out, static_cast<hipStream_t>(stream)), who);
}

}  // namespace

extern "C" {

a2d_status a2d_fix(int k, int64_t rows, int32_t hdim, int32_t out_dtype,
                   const float* const* O_parts, const float* const* m, const float* const* l,
                   void* O, float* lse, void* stream) {
  return fix_impl(k, rows, hdim, out_dtype, O_parts, m, l, O, a2d::plain_out(), lse, stream, "a2d_fix");
}

a2d_status a2d_attnfix(int k, int64_t rows, int32_t hdim, const float* const* O_parts, const float* const* m,
                       const float* const* l, float* N_out, float* m_out, float* l_out, void* stream) {
  const char* who = "a2d_attnfix";
  if (k < 1 || k > A2D_MAX_PARTS)
    return fail(A2D_ERR_INVALID_ARG, "%s: k=%d outside 1..%d", who, k, A2D_MAX_PARTS);
  if (rows < 1) return fail(A2D_ERR_INVALID_ARG, "%s: rows=%lld must be >= 1", who, (long long)rows);
  if (hdim < 4 || hdim % 4 != 0 || hdim > 1024)
    return fail(A2D_ERR_UNSUPPORTED, "%s: hdim=%d must be a multiple of 4 in 4..1024", who, hdim);
  if (rows * (int64_t)(hdim / 4) > ((int64_t)1 << 39))
    return fail(A2D_ERR_INVALID_ARG, "%s: rows * hdim too large", who);
  if (!O_parts || !m || !l) return fail(A2D_ERR_INVALID_ARG, "%s: pointer array is NULL", who);
  A2D_TRY(check_ptr(N_out, who, "N_out"));
  A2D_TRY(check_ptr(m_out, who, "m_out"));
  A2D_TRY(check_ptr(l_out, who, "l_out"));
  a2d::FixPtrs p;
  memset(&p, 0, sizeof(p));
  for (int x = 0; x < k; ++x) {
    A2D_TRY(check_ptr(O_parts[x], who, "O_parts[x]"));
    A2D_TRY(check_ptr(m[x], who, "m[x]"));
    A2D_TRY(check_ptr(l[x], who, "l[x]"));
    // a row's column groups are read by several lanes and written by others: no output may be an input
    if (O_parts[x] == N_out || m[x] == m_out || l[x] == l_out)
      return fail(A2D_ERR_INVALID_ARG, "%s: output %d aliases an input (the merge is not in place)", who, x);
    p.o[x] = O_parts[x]; p.m[x] = m[x]; p.l[x] = l[x];
  }
  a2d::trace_mark(static_cast<hipStream_t>(stream));
  return hip_result(a2d::launch_attnfix(k, rows, hdim, p, N_out, m_out, l_out, static_cast<hipStream_t>(stream)), who);
}

a2d_status a2d_fix_strided(int k, int32_t heads, int32_t nq, int32_t hdim, int32_t out_dtype,
                           const float* const* O_parts, const float* const* m, const float* const* l,
                           void* O, const a2d_layout* lo, float* lse, void* stream) {
  const char* who = "a2d_fix_strided";
  if (heads < 1 || nq < 1) return fail(A2D_ERR_INVALID_ARG, "%s: heads=%d nq=%d must be >= 1", who, heads, nq);
  a2d::OutMap om;
  A2D_TRY(out_map(lo, nq, hdim, out_dtype, who, &om));
  return fix_impl(k, (int64_t)heads * nq, hdim, out_dtype, O_parts, m, l, O, om, lse, stream, who);
}

a2d_status a2d_fix_bwd_strided(int k, int32_t heads, int32_t rows, int32_t hdim, int32_t out_dtype,
                               const float* const* parts, void* out, const a2d_layout* lout, void* stream) {
  const char* who = "a2d_fix_bwd_strided";
  if (heads < 1 || rows < 1) return fail(A2D_ERR_INVALID_ARG, "%s: heads=%d rows=%d must be >= 1", who, heads, rows);
  if (hdim < 4 || hdim % 4 != 0 || hdim > 1024)
    return fail(A2D_ERR_UNSUPPORTED, "%s: hdim=%d must be a multiple of 4 in 4..1024", who, hdim);
  a2d::OutMap om;
  A2D_TRY(out_map(lout, rows, hdim, out_dtype, who, &om));
  return fix_bwd_impl(k, (int64_t)heads * rows * hdim, hdim, out_dtype, parts, out, om, stream, who);
}

a2d_status a2d_partial_bwd_seg(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, const void* O,
                               const void* dO, const float* lse, float* dQ_part, float* dK_part,
                               float* dV_part, void* workspace, size_t workspace_bytes,
                               void* stream) {
  const char* who = "a2d_partial_bwd_seg";
  A2D_TRY(check_desc(desc, who));
  a2d::SegList g;
  A2D_TRY(make_segments(desc, nseg, segs, who, &g));
  return partial_bwd_impl(desc, g, Q, K, V, O, dO, lse, dQ_part, dK_part, dV_part, workspace,
                          workspace_bytes, stream, who);
}

a2d_status a2d_partial_bwd_acc(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, const void* O,
                               const void* dO, const float* lse, float* dQ_part, float* dK_part,
                               float* dV_part, void* workspace, size_t workspace_bytes,
                               void* stream) {
  const char* who = "a2d_partial_bwd_acc";
  A2D_TRY(check_desc(desc, who));
  a2d::SegList g = one_segment(desc);
  if (nseg != 0) A2D_TRY(make_segments(desc, nseg, segs, who, &g));
  g.acc = 1;
  return partial_bwd_impl(desc, g, Q, K, V, O, dO, lse, dQ_part, dK_part, dV_part, workspace,
                          workspace_bytes, stream, who);
}

a2d_status a2d_partial_bwd(const a2d_tile_desc* desc, const void* Q, const void* K, const void* V,
                           const void* O, const void* dO, const float* lse, float* dQ_part,
                           float* dK_part, float* dV_part, void* workspace, size_t workspace_bytes,
                           void* stream) {
  const char* who = "a2d_partial_bwd";
  A2D_TRY(check_desc(desc, who));
  return partial_bwd_impl(desc, one_segment(desc), Q, K, V, O, dO, lse, dQ_part, dK_part, dV_part,
                          workspace, workspace_bytes, stream, who);
}

a2d_status a2d_fix_bwd(int k, int64_t n, int32_t out_dtype, const float* const* parts, void* out,
                       void* stream) {
  return fix_bwd_impl(k, n, 4, out_dtype, parts, out, a2d::plain_out(), stream, "a2d_fix_bwd");
}

const char* a2d_status_str(a2d_status status) {
  switch (status) {
    case A2D_OK: return "ok";
    case A2D_ERR_INVALID_ARG: return "invalid argument";
    case A2D_ERR_UNSUPPORTED: return "unsupported dtype or shape";
    case A2D_ERR_MISALIGNED: return "misaligned pointer";
    case A2D_ERR_WORKSPACE: return "workspace missing or too small";
    case A2D_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

size_t a2d_mfma_ceiling_scratch_bytes(void) {
  int cus = 0;
  if (a2d::device_cus(&cus) != hipSuccess) return 0;
  // four workgroups per compute unit: enough wavefronts to keep every SIMD's MFMA pipe full
  // however the dispatcher spreads them
  return (size_t)4 * cus * a2d::mfma_probe_threads() * sizeof(float) + 16;
}

namespace {
// runs one of the probes twice (the first run settles the clocks) and converts its counters.
// mode 0 / 1: MFMA only, constant / random operands; 2: forward loop model; 3: dK/dV loop model
// (arg = parts left out); 4: LDS reads (arg = kind).  *rate: TFLOP/s, or TB/s for mode 4.
a2d_status run_probe(const char* who, int iters, int mode, int arg, void* scratch, size_t scratch_bytes, double* rate,
                     double* shader_mhz) {
  if (iters < 1 || iters > (1 << 22)) return fail(A2D_ERR_INVALID_ARG, "%s: iters=%d outside 1..2^22", who, iters);
  if (!rate || !shader_mhz) return fail(A2D_ERR_INVALID_ARG, "%s: result pointer is NULL", who);
  A2D_TRY(check_ptr(scratch, who, "scratch"));
  const size_t need = a2d_mfma_ceiling_scratch_bytes();
  if (need == 0) return fail(A2D_ERR_HIP, "%s: cannot query the device", who);
  if (scratch_bytes < need)
    return fail(A2D_ERR_WORKSPACE, "%s: scratch of %zu bytes, %zu needed", who, scratch_bytes, need);
  // MFMA-only probe: four workgroups per compute unit; the others: one (64 / 96 KiB of LDS each)
  const int all = (int)((need - 16) / (a2d::mfma_probe_threads() * sizeof(float)));
  const int blocks = mode >= 2 ? all / 4 : all;
  float* sc = static_cast<float*>(scratch);
  auto launch = [&]() {
    return mode == 4   ? a2d::launch_lds_read_probe(blocks, iters, arg, sc, nullptr)
           : mode == 3 ? a2d::launch_bwd_mix_probe(blocks, iters, arg, sc, nullptr)
           : mode == 2 ? a2d::launch_mix_probe(blocks, iters, sc, nullptr)
                       : a2d::launch_mfma_probe(blocks, iters, mode, sc, nullptr);
  };
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return fail(A2D_ERR_HIP, "%s: hipEventCreate failed", who);
  hipError_t e = launch();   // warm-up, clocks settle
  if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
  if (e == hipSuccess) e = hipEventRecord(e0, nullptr);
  if (e == hipSuccess) e = launch();
  if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  unsigned long long clocks[2] = {0, 0};
  if (e == hipSuccess)
    e = hipMemcpy(clocks, sc + (size_t)blocks * a2d::mfma_probe_threads(), sizeof(clocks), hipMemcpyDeviceToHost);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return hip_result(e, who);
  // every wavefront issues iters * 16 MFMAs of 2 * 32 * 32 * 16 flop - or 16 LDS reads of 1 KiB
  // (a transposing read counts as its two 512-byte halves); 8 wavefronts per workgroup
  const double units = (double)blocks * (a2d::mfma_probe_threads() / 64) * iters * a2d::mfma_probe_mfma_per_iter();
  *rate = units * (mode == 4 ? 1024.0 : 2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
  *shader_mhz = clocks[1] ? (double)clocks[0] / ((double)clocks[1] / 100.0) : 0.0;   // 100 MHz wall counter
  return A2D_OK;
}
}  // namespace

a2d_status a2d_mfma_ceiling(int iters, int random_data, void* scratch, size_t scratch_bytes,
                            double* tflops, double* shader_mhz) {
  return run_probe("a2d_mfma_ceiling", iters, random_data ? 1 : 0, 0, scratch, scratch_bytes, tflops, shader_mhz);
}

a2d_status a2d_forward_mix_ceiling(int iters, void* scratch, size_t scratch_bytes, double* tflops,
                                   double* shader_mhz) {
  return run_probe("a2d_forward_mix_ceiling", iters, 2, 0, scratch, scratch_bytes, tflops, shader_mhz);
}

a2d_status a2d_backward_mix_ceiling(int iters, int leave_out, void* scratch, size_t scratch_bytes, double* tflops,
                                    double* shader_mhz) {
  const char* who = "a2d_backward_mix_ceiling";
  if (leave_out < 0 || leave_out > 7 || ((leave_out & 4) && !(leave_out & 1)))
    return fail(A2D_ERR_INVALID_ARG, "%s: leave_out=%d (bits 0..2; the barrier only together with the mailbox)", who,
                leave_out);
  if (leave_out == 4 || leave_out == 6) return fail(A2D_ERR_INVALID_ARG, "%s: leave_out=%d", who, leave_out);
  return run_probe(who, iters, 3, leave_out, scratch, scratch_bytes, tflops, shader_mhz);
}

a2d_status a2d_lds_read_ceiling(int iters, int transposing, void* scratch, size_t scratch_bytes, double* tbytes_per_s,
                                double* shader_mhz) {
  return run_probe("a2d_lds_read_ceiling", iters, 4, transposing ? 1 : 0, scratch, scratch_bytes, tbytes_per_s,
                   shader_mhz);
}

void a2d_debug_force_generic(int on) { a2d::set_force_generic(on != 0); }

void a2d_debug_trace(void** events, int n) { a2d::trace_set(reinterpret_cast<hipEvent_t*>(events), n); }

int a2d_debug_trace_count(void) { return a2d::trace_count(); }

a2d_status a2d_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  const char* who = "a2d_copy_probe";
  A2D_TRY(check_ptr(dst, who, "dst"));
  A2D_TRY(check_ptr(src, who, "src"));
  if (bytes < 16 || bytes % 16 != 0)
    return fail(A2D_ERR_INVALID_ARG, "%s: bytes=%zu must be a positive multiple of 16", who, bytes);
  return hip_result(a2d::launch_copy_probe(dst, src, bytes / 16, static_cast<hipStream_t>(stream)), who);
}

const char* a2d_last_error(void) { return g_err; }

const char* a2d_version(void) { return "0.1"; }

}  // extern "C"
