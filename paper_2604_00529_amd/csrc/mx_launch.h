// Host-side declarations shared by the C-ABI layer (mx_api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mx.h"

namespace mx {

// Status of the launch just made; a failure is reported on stderr with the runtime's own message.
mx_status_t launch_status(const char* what);

// One tensor of a Slice-and-Scale launch (device pointers): one anchor, up to kSsMaxTargets targets
// converted in the same pass.
constexpr int kSsMaxTargets = 3;
struct SsTensor {
  const void* codes_h;
  const uint8_t* scales_h;
  void* codes_l[kSsMaxTargets];
  uint8_t* scales_l[kSsMaxTargets];
  int64_t nblocks;
};

constexpr int kSsLanes = 64;       // one wave per workgroup, one load per lane
// Workgroups per segment of a batched launch, as a shift.  Large segments keep a descriptor in the
// scalar caches over many workgroups; small ones bound the padding when tensors are small.
constexpr int kSsSegShiftLarge = 10, kSsSegShiftSmall = 7;

// One segment of a batched launch: kind 0 = `count` code pieces, kind 1 = `count` scale bytes.
struct SsSegment {
  const void* in;
  void* out[kSsMaxTargets];
  int64_t count;
  int32_t kind;
  int32_t pad;
  int64_t pad2[2];                 // 64 bytes: one descriptor per scalar cache line
};

// Tensor descriptors travel to the segment-table writer as kernel arguments (nothing is copied from
// host memory that would have to outlive the call), as many per launch as 4 KiB of arguments hold.
// One tensor takes 4 + 2 * n_targets words: codes_h, scales_h, nblocks, first code segment | first
// scale segment << 32 (relative to the chunk), then codes_l[q], then scales_l[q].
constexpr int kSsChunkWords = 496;
struct SsChunk {
  int64_t w[kSsChunkWords];
  int32_t count, n_targets;
  int64_t seg0;                    // first segment of the chunk in the launch
};

// The target list of one launch: element ids in increasing enum order, -1 = unused slot.
struct SsTargets {
  int elem[kSsMaxTargets];
  int bits[kSsMaxTargets];
  int n;
};

// The tensors of a batched launch, read from the caller's descriptor arrays where they lie (nothing is copied):
// targets[i * n_targets + q] is target q of anchor i.
struct SsBatch {
  const mx_packed_t* anchors;
  const mx_packed_t* targets;
  int n, n_targets;
  SsTensor tensor(int i) const {
    SsTensor t{};
    t.codes_h = anchors[i].codes;
    t.scales_h = anchors[i].scales;
    t.nblocks = anchors[i].outer * anchors[i].nblocks;
    for (int q = 0; q < n_targets; ++q) {
      t.codes_l[q] = targets[(size_t)i * n_targets + q].codes;
      t.scales_l[q] = targets[(size_t)i * n_targets + q].scales;
    }
    return t;
  }
};

// Segment descriptors of the library's own table (64 bytes each: 1 MiB per GPU): see mx_slice_and_scale_batched_noalloc.
constexpr int kSsStaticSegments = 16384;
// Address and size, on the current device, of that table.
mx_status_t ss_static_workspace(void** ptr, size_t* bytes);

mx_status_t ss_launch_one(int anchor, const SsTargets& tg, bool hw, const SsTensor& t, int block, int tie, hipStream_t stream);
size_t ss_workspace_bytes(int n, int64_t total_blocks);
mx_status_t ss_launch_many(int anchor, const SsTargets& tg, bool hw, const SsBatch& batch, int block, void* workspace,
                           size_t workspace_bytes, int tie, hipStream_t stream);

// Dense <-> packed kernels.  `dense` / `ld` in elements of dtype; outer / nblocks as in mx.h.
struct DenseArg {
  void* data;
  int dtype;
  int64_t rows, cols, ld;
};
mx_status_t quantize_launch(int elem, int axis, int block, int tie, const DenseArg& src, void* codes, uint8_t* scales,
                            hipStream_t stream);
mx_status_t dequant_launch(int elem, int axis, int block, const void* codes, const uint8_t* scales, const DenseArg& dst,
                           hipStream_t stream);
mx_status_t fake_quant_launch(int target, int anchor /* -1: none */, int axis, int block, int tie, const DenseArg& src,
                              const DenseArg& dst, hipStream_t stream);

mx_status_t gemm_ss_fp4_launch(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                               const uint8_t* w_scales, float* c, int64_t M, int64_t N, int64_t K, int64_t ldc,
                               hipStream_t stream);
bool gemm_hoist_pays(int64_t M, int64_t N);
int gemm_splitk_slices(int64_t M, int64_t N, int64_t K, size_t workspace_bytes, int* ntw_out);
bool gemm_ss_fp4_splitk(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                        float* c, int64_t M, int64_t N, int64_t K, int64_t ldc, void* workspace, size_t workspace_bytes,
                        hipStream_t stream, mx_status_t* status);
bool gemm_fp8_fp4_splitk(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w4_codes, const uint8_t* w4_scales,
                         float* c, int64_t M, int64_t N, int64_t K, int64_t ldc, void* workspace, size_t workspace_bytes,
                         hipStream_t stream, mx_status_t* status);
bool gemm_big_tiles_pay(int64_t M, int64_t N);
mx_status_t gemm_fp8_fp4_launch(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w4_codes,
                                const uint8_t* w4_scales, float* c, int64_t M, int64_t N, int64_t K, int64_t ldc,
                                hipStream_t stream);

}  // namespace mx
