// C-ABI layer: argument validation on the host, then dispatch to the kernel launchers.
// Nothing here allocates (host or device), frees or synchronizes; a call that fails validation launches nothing.
#include "mx_device.h"
#include "mx_launch.h"
#include <cstdio>

namespace {

struct ElemInfo {
  int bits, emax, family;  // family 0 = MXINT, 1 = MXFP
};

bool elem_info(int e, ElemInfo* out) {
  switch (e) {
#define MX_CASE(ID) \
  case ID:          \
    *out = ElemInfo{mx::Elem<ID>::bits, mx::Elem<ID>::emax, mx::Elem<ID>::is_int ? 0 : 1}; \
    return true;
    MX_CASE(MX_INT8) MX_CASE(MX_INT7) MX_CASE(MX_INT6) MX_CASE(MX_INT5) MX_CASE(MX_INT4) MX_CASE(MX_INT3) MX_CASE(MX_INT2)
    MX_CASE(MX_FP8_E4M3) MX_CASE(MX_FP7_E3M3) MX_CASE(MX_FP6_E3M2) MX_CASE(MX_FP6_E2M3) MX_CASE(MX_FP5_E2M2)
    MX_CASE(MX_FP4_E2M1)
#undef MX_CASE
    default:
      return false;
  }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

mx_status_t check_format(const mx_format_t* f, ElemInfo* info) {
  if (!f) return MX_ERR_NULL;
  if (!elem_info((int)f->elem, info)) return MX_ERR_FORMAT;
  if (f->scale != MX_SCALE_E8M0) return MX_ERR_FORMAT;
  if ((int)f->round < MX_ROUND_DEFAULT || (int)f->round > MX_ROUND_HALF_EVEN) return MX_ERR_FORMAT;
  if (f->axis != 0 && f->axis != 1) return MX_ERR_SHAPE;
  if (f->block <= 0) return MX_ERR_SHAPE;
  if (f->block != 16 && f->block != 32 && f->block != 64 && f->block != 128) return MX_ERR_UNSUPPORTED;
  return MX_OK;
}

// outer / nblocks of a [rows, cols] tensor blocked along f->axis
mx_status_t blocked_shape(const mx_format_t* f, int64_t rows, int64_t cols, int64_t* outer, int64_t* nblocks) {
  if (rows < 0 || cols < 0) return MX_ERR_SHAPE;
  int64_t ext = f->axis == 1 ? cols : rows;
  if (ext % f->block) return MX_ERR_SHAPE;
  *outer = f->axis == 1 ? rows : cols;
  *nblocks = ext / f->block;
  return MX_OK;
}

mx_status_t check_dense(const mx_dense_t* d) {
  if (!d) return MX_ERR_NULL;
  if (d->dtype != MX_F32 && d->dtype != MX_BF16) return MX_ERR_FORMAT;
  if (d->rows < 0 || d->cols < 0 || d->ld < d->cols) return MX_ERR_SHAPE;
  if (d->rows > 0 && d->cols > 0 && !d->data) return MX_ERR_NULL;
  if (!aligned16(d->data) || (d->ld % 8)) return MX_ERR_ALIGN;
  return MX_OK;
}

mx_status_t check_packed(const mx_packed_t* p) {
  if (!p) return MX_ERR_NULL;
  if (p->outer < 0 || p->nblocks < 0) return MX_ERR_SHAPE;
  if (p->outer > 0 && p->nblocks > 0 && (!p->codes || !p->scales)) return MX_ERR_NULL;
  if (!aligned16(p->codes) || !aligned16(p->scales)) return MX_ERR_ALIGN;
  if (p->outer > 0 && p->nblocks > ((int64_t)1 << 40) / p->outer) return MX_ERR_UNSUPPORTED;
  return MX_OK;
}

// Blocks of 16: the row kernels pack and unpack codes in windows of 32, so a tensor with an odd number of such blocks
// ends in half a window.  Element widths of 8 and 4 bits keep every lane's share of a window inside whole bytes of its
// own; the other widths share dwords across the lanes of a window and would touch bytes past the end of the codes.
bool partial_window_unsupported(const mx_format_t* f, const ElemInfo& info, int64_t rows, int64_t cols) {
  return f->block == 16 && (rows * cols) % 32 != 0 && info.bits != 8 && info.bits != 4;
}

// The tie rule the kernels implement in hardware conversions: ties to even on an MXFP target.
bool hw_tie(const ElemInfo& info, mx_round_t r) {
  return info.family == 1 && (r == MX_ROUND_DEFAULT || r == MX_ROUND_HALF_EVEN);
}

mx_status_t check_ss_pair(const mx_format_t* fa, const mx_format_t* ft, ElemInfo* ia, ElemInfo* it) {
  mx_status_t st = check_format(fa, ia);
  if (st != MX_OK) return st;
  st = check_format(ft, it);
  if (st != MX_OK) return st;
  if (ia->family != it->family || it->bits >= ia->bits) return MX_ERR_FORMAT;  // not a down-conversion
  if (fa->block != ft->block) return MX_ERR_FORMAT;
  if (fa->round != ft->round) return MX_ERR_FORMAT;
  if (fa->elem != MX_INT8 && fa->elem != MX_FP8_E4M3) return MX_ERR_UNSUPPORTED;
  return MX_OK;
}

}  // namespace

// hipGetLastError() after a launch also reports an error that an earlier, unrelated runtime call of this thread left
// behind (another library's event query that was "not ready", for instance).  Every entry point drops such a stale
// error before its first launch, so that MX_ERR_LAUNCH always means one of this library's own launches failed.
static inline void drop_stale_error() { (void)hipGetLastError(); }

namespace mx {
mx_status_t launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return MX_OK;
  fprintf(stderr, "libmx: launch of %s failed: %s\n", what, hipGetErrorString(e));
  return MX_ERR_LAUNCH;
}
}  // namespace mx

extern "C" {

int mx_elem_bits(mx_elem_t elem) {
  ElemInfo i;
  return elem_info((int)elem, &i) ? i.bits : -1;
}

int mx_elem_emax(mx_elem_t elem) {
  ElemInfo i;
  return elem_info((int)elem, &i) ? i.emax : -1;
}

mx_status_t mx_packed_bytes(const mx_format_t* f, int64_t rows, int64_t cols, size_t* code_bytes, size_t* scale_bytes) {
  ElemInfo info;
  mx_status_t st = check_format(f, &info);
  if (st != MX_OK) return st;
  if (!code_bytes || !scale_bytes) return MX_ERR_NULL;
  int64_t outer, nblocks;
  st = blocked_shape(f, rows, cols, &outer, &nblocks);
  if (st != MX_OK) return st;
  *scale_bytes = (size_t)(outer * nblocks);
  *code_bytes = (size_t)(outer * nblocks) * (size_t)(f->block * info.bits / 8);
  return MX_OK;
}

mx_status_t mx_quantize(const mx_format_t* f, const mx_dense_t* src, const mx_packed_t* dst, void* stream) {
  ElemInfo info;
  mx_status_t st = check_format(f, &info);
  if (st != MX_OK) return st;
  if ((st = check_dense(src)) != MX_OK) return st;
  if ((st = check_packed(dst)) != MX_OK) return st;
  int64_t outer, nblocks;
  if ((st = blocked_shape(f, src->rows, src->cols, &outer, &nblocks)) != MX_OK) return st;
  if (outer != dst->outer || nblocks != dst->nblocks) return MX_ERR_SHAPE;
  if (outer == 0 || nblocks == 0) return MX_OK;
  if (partial_window_unsupported(f, info, src->rows, src->cols)) return MX_ERR_UNSUPPORTED;
  mx::DenseArg s{src->data, (int)src->dtype, src->rows, src->cols, src->ld};
  drop_stale_error();
  return mx::quantize_launch((int)f->elem, f->axis, f->block, (int)f->round, s, dst->codes, dst->scales, static_cast<hipStream_t>(stream));
}

// Validate an anchor format with n target formats; fill the launch's target list.
static mx_status_t check_ss_targets(const mx_format_t* fa, int32_t n_targets, const mx_format_t* fts, mx::SsTargets* tg,
                                    bool* hw) {
  if (!fts) return MX_ERR_NULL;
  if (n_targets < 1 || n_targets > mx::kSsMaxTargets) return MX_ERR_UNSUPPORTED;
  tg->n = n_targets;
  *hw = true;
  for (int q = 0; q < mx::kSsMaxTargets; ++q) { tg->elem[q] = -1; tg->bits[q] = 0; }
  for (int32_t q = 0; q < n_targets; ++q) {
    ElemInfo ia, it;
    mx_status_t st = check_ss_pair(fa, &fts[q], &ia, &it);
    if (st != MX_OK) return st;
    if (q > 0 && (int)fts[q].elem <= (int)fts[q - 1].elem) return MX_ERR_UNSUPPORTED;   // increasing enum order
    if (fts[q].round != fts[0].round) return MX_ERR_FORMAT;
    tg->elem[q] = (int)fts[q].elem;
    tg->bits[q] = it.bits;
    *hw = *hw && hw_tie(it, fts[q].round);
  }
  return MX_OK;
}

mx_status_t mx_slice_and_scale_multi(const mx_format_t* fa, const mx_packed_t* anchor, int32_t n_targets,
                                     const mx_format_t* fts, const mx_packed_t* targets, void* stream) {
  mx::SsTargets tg;
  bool hw;
  mx_status_t st = check_ss_targets(fa, n_targets, fts, &tg, &hw);
  if (st != MX_OK) return st;
  if (!targets) return MX_ERR_NULL;
  if ((st = check_packed(anchor)) != MX_OK) return st;
  int64_t nb = anchor->outer * anchor->nblocks;
  mx::SsTensor t{};
  t.codes_h = anchor->codes; t.scales_h = anchor->scales; t.nblocks = nb;
  for (int32_t q = 0; q < n_targets; ++q) {
    if ((st = check_packed(&targets[q])) != MX_OK) return st;
    if (nb != targets[q].outer * targets[q].nblocks) return MX_ERR_SHAPE;
    t.codes_l[q] = targets[q].codes; t.scales_l[q] = targets[q].scales;
  }
  if (nb == 0) return MX_OK;
  drop_stale_error();
  return mx::ss_launch_one((int)fa->elem, tg, hw, t, fa->block, (int)fts[0].round, static_cast<hipStream_t>(stream));
}

mx_status_t mx_slice_and_scale(const mx_format_t* fa, const mx_packed_t* anchor, const mx_format_t* ft,
                               const mx_packed_t* target, void* stream) {
  if (!ft) return MX_ERR_NULL;
  return mx_slice_and_scale_multi(fa, anchor, 1, ft, target, stream);
}

size_t mx_slice_and_scale_batched_workspace(int32_t n, int64_t total_blocks) {
  if (n <= 0 || total_blocks < 0) return 0;
  return mx::ss_workspace_bytes(n, total_blocks);
}

// Validation shared by the batched entry points: every descriptor is checked before anything is launched.
static mx_status_t check_ss_batch(int32_t n_targets, int32_t n, const mx_packed_t* anchors, const mx_packed_t* targets) {
  mx_status_t st;
  for (int32_t i = 0; i < n; ++i) {
    if ((st = check_packed(&anchors[i])) != MX_OK) return st;
    const int64_t nb = anchors[i].outer * anchors[i].nblocks;
    for (int32_t q = 0; q < n_targets; ++q) {
      const mx_packed_t* tq = &targets[(size_t)i * n_targets + q];
      if ((st = check_packed(tq)) != MX_OK) return st;
      if (nb != tq->outer * tq->nblocks) return MX_ERR_SHAPE;
    }
  }
  return MX_OK;
}

mx_status_t mx_slice_and_scale_multi_batched(const mx_format_t* fa, int32_t n_targets, const mx_format_t* fts, int32_t n,
                                             const mx_packed_t* anchors, const mx_packed_t* targets, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  mx::SsTargets tg;
  bool hw;
  mx_status_t st = check_ss_targets(fa, n_targets, fts, &tg, &hw);
  if (st != MX_OK) return st;
  if (n < 0) return MX_ERR_SHAPE;
  if (n == 0) return MX_OK;
  if (!anchors || !targets || !workspace) return MX_ERR_NULL;
  if (!aligned16(workspace)) return MX_ERR_ALIGN;
  if ((st = check_ss_batch(n_targets, n, anchors, targets)) != MX_OK) return st;
  drop_stale_error();
  return mx::ss_launch_many((int)fa->elem, tg, hw, mx::SsBatch{anchors, targets, n, n_targets}, fa->block, workspace, workspace_bytes,
                            (int)fts[0].round, static_cast<hipStream_t>(stream));
}

mx_status_t mx_slice_and_scale_batched(const mx_format_t* fa, const mx_format_t* ft, int32_t n, const mx_packed_t* anchors,
                                       const mx_packed_t* targets, void* workspace, size_t workspace_bytes, void* stream) {
  if (!ft) return MX_ERR_NULL;
  return mx_slice_and_scale_multi_batched(fa, 1, ft, n, anchors, targets, workspace, workspace_bytes, stream);
}

mx_status_t mx_slice_and_scale_batched_noalloc(const mx_format_t* fa, const mx_format_t* ft, int32_t n, const mx_packed_t* anchors,
                                               const mx_packed_t* targets, void* stream) {
  if (!ft) return MX_ERR_NULL;
  mx::SsTargets tg;
  bool hw;
  mx_status_t st = check_ss_targets(fa, 1, ft, &tg, &hw);
  if (st != MX_OK) return st;
  if (n < 0) return MX_ERR_SHAPE;
  if (n == 0) return MX_OK;
  if (!anchors || !targets) return MX_ERR_NULL;
  if ((st = check_ss_batch(1, n, anchors, targets)) != MX_OK) return st;
  drop_stale_error();
  void* table = nullptr;
  size_t table_bytes = 0;
  if ((st = mx::ss_static_workspace(&table, &table_bytes)) != MX_OK) return st;
  // (a launch that needs more segments than the table holds comes back as MX_ERR_WORKSPACE before anything is enqueued)
  return mx::ss_launch_many((int)fa->elem, tg, hw, mx::SsBatch{anchors, targets, n, 1}, fa->block, table, table_bytes, (int)ft->round,
                            static_cast<hipStream_t>(stream));
}

mx_status_t mx_fake_quant(const mx_format_t* target, const mx_format_t* anchor, const mx_dense_t* src, const mx_dense_t* dst,
                          void* stream) {
  ElemInfo it, ia;
  mx_status_t st = check_format(target, &it);
  if (st != MX_OK) return st;
  int anchor_elem = -1;
  if (anchor) {
    if ((st = check_format(anchor, &ia)) != MX_OK) return st;
    if (ia.family != it.family || it.bits >= ia.bits) return MX_ERR_FORMAT;
    if (anchor->block != target->block || anchor->axis != target->axis || anchor->round != target->round) return MX_ERR_FORMAT;
    if (anchor->elem != MX_INT8 && anchor->elem != MX_FP8_E4M3) return MX_ERR_UNSUPPORTED;
    anchor_elem = (int)anchor->elem;
  }
  if ((st = check_dense(src)) != MX_OK) return st;
  if ((st = check_dense(dst)) != MX_OK) return st;
  if (src->rows != dst->rows || src->cols != dst->cols) return MX_ERR_SHAPE;
  if (src->dtype != dst->dtype) return MX_ERR_UNSUPPORTED;
  if (src->data == dst->data && src->ld != dst->ld) return MX_ERR_SHAPE;
  int64_t outer, nblocks;
  if ((st = blocked_shape(target, src->rows, src->cols, &outer, &nblocks)) != MX_OK) return st;
  if (outer == 0 || nblocks == 0) return MX_OK;
  mx::DenseArg s{src->data, (int)src->dtype, src->rows, src->cols, src->ld};
  mx::DenseArg d{dst->data, (int)dst->dtype, dst->rows, dst->cols, dst->ld};
  drop_stale_error();
  return mx::fake_quant_launch((int)target->elem, anchor_elem, target->axis, target->block, (int)target->round, s, d,
                               static_cast<hipStream_t>(stream));
}

mx_status_t mx_dequant(const mx_format_t* f, const mx_packed_t* src, const mx_dense_t* dst, void* stream) {
  ElemInfo info;
  mx_status_t st = check_format(f, &info);
  if (st != MX_OK) return st;
  if ((st = check_packed(src)) != MX_OK) return st;
  if ((st = check_dense(dst)) != MX_OK) return st;
  int64_t outer, nblocks;
  if ((st = blocked_shape(f, dst->rows, dst->cols, &outer, &nblocks)) != MX_OK) return st;
  if (outer != src->outer || nblocks != src->nblocks) return MX_ERR_SHAPE;
  if (outer == 0 || nblocks == 0) return MX_OK;
  if (partial_window_unsupported(f, info, dst->rows, dst->cols)) return MX_ERR_UNSUPPORTED;
  mx::DenseArg d{dst->data, (int)dst->dtype, dst->rows, dst->cols, dst->ld};
  drop_stale_error();
  return mx::dequant_launch((int)f->elem, f->axis, f->block, src->codes, src->scales, d, static_cast<hipStream_t>(stream));
}

mx_status_t mx_gemm_ss_fp4(const mx_packed_t* a, const mx_packed_t* w_anchor, const mx_dense_t* c, void* stream) {
  mx_status_t st;
  if ((st = check_packed(a)) != MX_OK) return st;
  if ((st = check_packed(w_anchor)) != MX_OK) return st;
  if ((st = check_dense(c)) != MX_OK) return st;
  if (c->dtype != MX_F32) return MX_ERR_UNSUPPORTED;
  if (a->nblocks != w_anchor->nblocks || c->rows != a->outer || c->cols != w_anchor->outer) return MX_ERR_SHAPE;
  if (c->rows == 0 || c->cols == 0) return MX_OK;
  const int64_t K = a->nblocks * 32;
  if (K == 0 || K % 128 != 0 || K > 0x7FFFFFFF || c->rows > 0x7FFFFFFF || c->cols > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  drop_stale_error();
  return mx::gemm_ss_fp4_launch(static_cast<const uint8_t*>(a->codes), a->scales, static_cast<const uint8_t*>(w_anchor->codes),
                                w_anchor->scales, static_cast<float*>(c->data), c->rows, c->cols, K, c->ld,
                                static_cast<hipStream_t>(stream));
}

size_t mx_gemm_ss_fp4_workspace(int64_t n, int64_t k) {
  if (n <= 0 || k <= 0 || k % 32 != 0) return 0;
  return (size_t)n * (size_t)k / 2 + (size_t)n * (size_t)k / 32;   // E2M1 codes, then their scale bytes
}

int mx_gemm_ss_fp4_ws_slices(int64_t m, int64_t n, int64_t k, size_t workspace_bytes) {
  if (m <= 0 || n <= 0 || k <= 0 || k % 128 != 0 || k > 0x7FFFFFFF || m > 0x7FFFFFFF || n > 0x7FFFFFFF) return 1;
  if (workspace_bytes < mx_gemm_ss_fp4_workspace(n, k)) return 1;
  if (m >= MX_GEMM_HOIST_MIN_ROWS && mx::gemm_hoist_pays(m, n)) return 1;
  return mx::gemm_splitk_slices(m, n, k, workspace_bytes, nullptr);
}

mx_status_t mx_gemm_ss_fp4_ws(const mx_packed_t* a, const mx_packed_t* w_anchor, const mx_dense_t* c, void* workspace,
                              size_t workspace_bytes, void* stream) {
  mx_status_t st;
  if ((st = check_packed(a)) != MX_OK) return st;
  if ((st = check_packed(w_anchor)) != MX_OK) return st;
  if ((st = check_dense(c)) != MX_OK) return st;
  if (!workspace) return mx_gemm_ss_fp4(a, w_anchor, c, stream);
  if (c->dtype != MX_F32) return MX_ERR_UNSUPPORTED;
  if (a->nblocks != w_anchor->nblocks || c->rows != a->outer || c->cols != w_anchor->outer) return MX_ERR_SHAPE;
  if (c->rows == 0 || c->cols == 0) return MX_OK;
  const int64_t K = a->nblocks * 32, N = w_anchor->outer;
  if (K == 0 || K % 128 != 0 || K > 0x7FFFFFFF || c->rows > 0x7FFFFFFF || N > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  if (!aligned16(workspace)) return MX_ERR_ALIGN;
  if (workspace_bytes < mx_gemm_ss_fp4_workspace(N, K)) return MX_ERR_WORKSPACE;
  if (c->rows < MX_GEMM_HOIST_MIN_ROWS || !mx::gemm_hoist_pays(c->rows, c->cols)) {
    // Few rows or too few tiles to fill the GPU: the kernels that slice on the fly -- with K split over several
    // workgroups per tile, their partial sums in the workspace, when the tiles alone leave most of the GPU idle.
    drop_stale_error();
    if (mx::gemm_ss_fp4_splitk(static_cast<const uint8_t*>(a->codes), a->scales, static_cast<const uint8_t*>(w_anchor->codes),
                               w_anchor->scales, static_cast<float*>(c->data), c->rows, N, K, c->ld, workspace, workspace_bytes,
                               static_cast<hipStream_t>(stream), &st))
      return st;
    return mx_gemm_ss_fp4(a, w_anchor, c, stream);
  }
  // W_t = Q_{A->t}(W_A) (Eq. (6)) once, by the Slice-and-Scale kernel, then the product
  uint8_t* w4 = static_cast<uint8_t*>(workspace);
  const mx_format_t fa = {MX_FP8_E4M3, MX_SCALE_E8M0, 32, 1, MX_ROUND_DEFAULT}, ft = {MX_FP4_E2M1, MX_SCALE_E8M0, 32, 1, MX_ROUND_DEFAULT};
  const mx_packed_t wt = {w4, w4 + (size_t)N * (size_t)K / 2, N, K / 32};
  if ((st = mx_slice_and_scale(&fa, w_anchor, &ft, &wt, stream)) != MX_OK) return st;
  return mx::gemm_fp8_fp4_launch(static_cast<const uint8_t*>(a->codes), a->scales, w4, wt.scales, static_cast<float*>(c->data),
                                 c->rows, N, K, c->ld, static_cast<hipStream_t>(stream));
}

// shared checks of the two entry points that multiply by a kept W_t; *k_out = K; MX_OK with *k_out = 0: nothing to do
static mx_status_t check_gemm_kept(const mx_packed_t* a, const mx_packed_t* w_t, const mx_dense_t* c, int64_t* k_out) {
  mx_status_t st;
  *k_out = 0;
  if ((st = check_packed(a)) != MX_OK) return st;
  if ((st = check_packed(w_t)) != MX_OK) return st;
  if ((st = check_dense(c)) != MX_OK) return st;
  if (c->dtype != MX_F32) return MX_ERR_UNSUPPORTED;
  if (a->nblocks != w_t->nblocks || c->rows != a->outer || c->cols != w_t->outer) return MX_ERR_SHAPE;
  if (c->rows == 0 || c->cols == 0) return MX_OK;
  const int64_t K = a->nblocks * 32;
  if (K == 0 || K % 128 != 0 || K > 0x7FFFFFFF || c->rows > 0x7FFFFFFF || c->cols > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  *k_out = K;
  return MX_OK;
}

mx_status_t mx_gemm_fp8_fp4(const mx_packed_t* a, const mx_packed_t* w_t, const mx_dense_t* c, void* stream) {
  int64_t K;
  mx_status_t st = check_gemm_kept(a, w_t, c, &K);
  if (st != MX_OK || K == 0) return st;
  drop_stale_error();
  return mx::gemm_fp8_fp4_launch(static_cast<const uint8_t*>(a->codes), a->scales, static_cast<const uint8_t*>(w_t->codes),
                                 w_t->scales, static_cast<float*>(c->data), c->rows, c->cols, K, c->ld,
                                 static_cast<hipStream_t>(stream));
}

static bool gemm_kept_shape_ok(int64_t m, int64_t n, int64_t k) {
  return m > 0 && n > 0 && k > 0 && k % 128 == 0 && k <= 0x7FFFFFFF && m <= 0x7FFFFFFF && n <= 0x7FFFFFFF;
}

int mx_gemm_fp8_fp4_ws_slices(int64_t m, int64_t n, int64_t k, size_t workspace_bytes) {
  if (!gemm_kept_shape_ok(m, n, k) || mx::gemm_big_tiles_pay(m, n)) return 1;
  return mx::gemm_splitk_slices(m, n, k, workspace_bytes, nullptr);
}

size_t mx_gemm_fp8_fp4_workspace(int64_t m, int64_t n, int64_t k) {
  const int slices = mx_gemm_fp8_fp4_ws_slices(m, n, k, ~(size_t)0);
  if (slices <= 1) return 0;
  return (size_t)slices * (size_t)m * (size_t)((n + 3) & ~(int64_t)3) * sizeof(float);   // the partial sums of the K slices
}

mx_status_t mx_gemm_fp8_fp4_ws(const mx_packed_t* a, const mx_packed_t* w_t, const mx_dense_t* c, void* workspace,
                               size_t workspace_bytes, void* stream) {
  int64_t K;
  mx_status_t st = check_gemm_kept(a, w_t, c, &K);
  if (st != MX_OK || K == 0) return st;
  if (!workspace || workspace_bytes == 0 || mx::gemm_big_tiles_pay(c->rows, c->cols)) return mx_gemm_fp8_fp4(a, w_t, c, stream);
  if (!aligned16(workspace)) return MX_ERR_ALIGN;
  drop_stale_error();
  if (mx::gemm_fp8_fp4_splitk(static_cast<const uint8_t*>(a->codes), a->scales, static_cast<const uint8_t*>(w_t->codes),
                              w_t->scales, static_cast<float*>(c->data), c->rows, c->cols, K, c->ld, workspace, workspace_bytes,
                              static_cast<hipStream_t>(stream), &st))
    return st;
  return mx_gemm_fp8_fp4(a, w_t, c, stream);
}

const char* mx_status_str(mx_status_t status) {
  switch (status) {
    case MX_OK: return "ok";
    case MX_ERR_NULL: return "null pointer";
    case MX_ERR_FORMAT: return "bad format";
    case MX_ERR_SHAPE: return "bad shape";
    case MX_ERR_ALIGN: return "bad alignment";
    case MX_ERR_UNSUPPORTED: return "unsupported";
    case MX_ERR_LAUNCH: return "launch failed";
    case MX_ERR_WORKSPACE: return "workspace too small";
  }
  return "unknown status";
}

}  // extern "C"
