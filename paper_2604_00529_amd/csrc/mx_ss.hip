// Slice-and-Scale kernels (Eq. (4) SSMXINT, Eq. (6) SSMXFP): 8-bit anchor -> narrower target.
//
// The packed layout is a flat run of blocks, so the conversion is a streaming map with no
// reduction and no neighbour dependence.  One lane converts one "piece" of CPL codes (16 = half
// a block for even target widths: one coalesced 128-bit load, one packed store; 32 = a whole
// block for odd widths).  The scale bytes are a second, independent stream (byte + De,
// saturating) handled by workgroups of their own at 16 bytes per lane.
//
// Launch shape, from measurement on MI355X: single-wave workgroups that each issue ONE load per
// lane and exit.  The dispatcher then keeps the set of in-flight waves on a narrow, advancing
// front of addresses, which HBM serves far better than unrolled or looping (persistent) waves.
#include "mx_device.h"
#include "mx_launch.h"

namespace mx {

// ---- one piece: CPL anchor codes (CPL/4 dwords) -> CPL * bits / 32 dwords
template <int ANCHOR, int TARGET, bool HW, int CPL>
__device__ __forceinline__ void slice_piece(const uint32_t (&in)[CPL / 4], uint32_t (&out)[CPL * Elem<TARGET>::bits / 32],
                                            int tie) {
  using T = Elem<TARGET>;
  constexpr int NIN = CPL / 4;
  if constexpr (Elem<ANCHOR>::is_int) {
    uint32_t c[NIN];
#pragma unroll
    for (int i = 0; i < NIN; ++i) c[i] = slice_int8x4<T::bits>(in[i], tie);
    pack_bytes<T::bits, NIN>(c, out);
  } else {
    constexpr int DE = Elem<ANCHOR>::emax - T::emax;
    const float two_de = __uint_as_float((uint32_t)(127 + DE) << 23);
    if constexpr (HW && T::hw == HW_FP4) {
      // E4M3 -> fp32 (exact) -> E2M1 with the 2^De division folded into the conversion's scale
#pragma unroll
      for (int j = 0; j < NIN / 2; ++j) {
        uint32_t w = 0;
        static_for<0, 2>([&](auto hh) {
          constexpr int H = decltype(hh)::value;
          uint32_t x = e4m3_nan_to_max(in[2 * j + H]);
          f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(x, false);
          f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(x, true);
          w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, lo.x, lo.y, two_de, 2 * H);
          w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, hi.x, hi.y, two_de, 2 * H + 1);
        });
        out[j] = w;
      }
    } else if constexpr (HW && (T::hw == HW_FP6 || T::hw == HW_BF6)) {
      // E4M3 -> fp16 (exact: 4 significant bits, exponents -9..8) -> FP6 codes, 32 at a time
      f16x32 h = {};
      const float one = __uint_as_float(127u << 23);
#pragma unroll
      for (int i = 0; i < NIN; ++i) {
        uint32_t x = e4m3_nan_to_max(in[i]);
        f16x2 a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(x, one, false);
        f16x2 b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(x, one, true);
        h[4 * i] = a.x; h[4 * i + 1] = a.y; h[4 * i + 2] = b.x; h[4 * i + 3] = b.y;
      }
      u32x6 p = cvt_pk32_fp6_f16<T::hw == HW_BF6>(h, two_de);
#pragma unroll
      for (int i = 0; i < CPL * 6 / 32; ++i) out[i] = p[i];
    } else {
      uint32_t c[NIN];
#pragma unroll
      for (int i = 0; i < NIN; ++i) {
        uint32_t x = e4m3_nan_to_max(in[i]);
        uint32_t r = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) r |= slice_e4m3_sw<TARGET>((x >> (8 * b)) & 0xFFu, tie) << (8 * b);
        c[i] = r;
      }
      pack_bytes<T::bits, NIN>(c, out);
    }
  }
}

// codes per lane: half a block when that ends on a dword boundary, else a whole block
template <int TARGET>
struct Piece { static constexpr int cpl = (Elem<TARGET>::bits % 2 == 0) ? 16 : 32; };

// ---- piece p of a run of pieces: load, convert, store
template <int ANCHOR, int TARGET, bool HW>
__device__ __forceinline__ void ss_piece(const void* __restrict__ in, void* __restrict__ out, int64_t p, int tie) {
  constexpr int CPL = Piece<TARGET>::cpl, NIN = CPL / 4, NOUT = CPL * Elem<TARGET>::bits / 32;
  uint32_t x[NIN], y[NOUT];
  const u32x4* src = reinterpret_cast<const u32x4*>(in) + p * (NIN / 4);
#pragma unroll
  for (int i = 0; i < NIN / 4; ++i) {
    u32x4 t = __builtin_nontemporal_load(src + i);
    x[4 * i] = t.x; x[4 * i + 1] = t.y; x[4 * i + 2] = t.z; x[4 * i + 3] = t.w;
  }
  slice_piece<ANCHOR, TARGET, HW, CPL>(x, y, tie);
  store_dwords<NOUT>(reinterpret_cast<uint32_t*>(out) + p * NOUT, y);
}

// ---- 16 scale bytes per lane
template <int DE>
__device__ __forceinline__ void ss_scale_chunk(const uint8_t* __restrict__ sh, uint8_t* __restrict__ sl, int64_t chunk,
                                               int64_t nbytes) {
  int64_t i0 = chunk * 16;
  if (i0 + 16 <= nbytes) {
    u32x4 v = *reinterpret_cast<const u32x4*>(sh + i0);
    v.x = scale_add_x4(v.x, DE); v.y = scale_add_x4(v.y, DE); v.z = scale_add_x4(v.z, DE); v.w = scale_add_x4(v.w, DE);
    *reinterpret_cast<u32x4*>(sl + i0) = v;
  } else {
    for (int64_t i = i0; i < nbytes; ++i) {
      uint32_t b = sh[i];
      sl[i] = (uint8_t)(b == 255u ? 255u : (b + DE > 254u ? 254u : b + DE));
    }
  }
}

// ---- one tensor: workgroups [0, code_wgs) convert pieces, the rest scale bytes
template <int ANCHOR, int TARGET, bool HW>
__global__ __launch_bounds__(kSsLanes) void ss_kernel(const void* __restrict__ ch, const uint8_t* __restrict__ sh,
                                                      void* __restrict__ cl, uint8_t* __restrict__ sl, int64_t nblocks,
                                                      int64_t code_wgs, int tie) {
  constexpr int DE = Elem<ANCHOR>::emax - Elem<TARGET>::emax;
  constexpr int CPL = Piece<TARGET>::cpl;
  int64_t wg = blockIdx.x;
  if (wg < code_wgs) {
    int64_t p = wg * kSsLanes + threadIdx.x;
    if (p < nblocks * (32 / CPL)) ss_piece<ANCHOR, TARGET, HW>(ch, cl, p, tie);
  } else {
    int64_t c = (wg - code_wgs) * kSsLanes + threadIdx.x;
    if (c * 16 < nblocks) ss_scale_chunk<DE>(sh, sl, c, nblocks);
  }
}

// ---- many tensors in one launch.  The work is cut into fixed-size segments (kSsSegWgs
// workgroups each), so a workgroup finds its segment with a shift and needs ONE dependent
// scalar load (the 32-byte segment descriptor) before its data load.
template <int ANCHOR, int TARGET, bool HW>
__global__ __launch_bounds__(kSsLanes) void ss_batched_kernel(const SsSegment* __restrict__ segs, int tie) {
  constexpr int DE = Elem<ANCHOR>::emax - Elem<TARGET>::emax;
  const SsSegment s = segs[blockIdx.x / kSsSegWgs];
  int64_t item = (int64_t)(blockIdx.x % kSsSegWgs) * kSsLanes + threadIdx.x;
  if (s.kind == 0) {
    if (item < s.count) ss_piece<ANCHOR, TARGET, HW>(s.in, s.out, item, tie);
  } else {
    if (item * 16 < s.count) ss_scale_chunk<DE>(static_cast<const uint8_t*>(s.in), static_cast<uint8_t*>(s.out), item, s.count);
  }
}

// Tensor table from kernel arguments into device memory (no host buffer has to outlive the call).
__global__ void ss_table_kernel(SsTableChunk chunk, SsTensor* __restrict__ table) {
  int i = threadIdx.x;
  if (i < chunk.count) table[chunk.base + i] = chunk.t[i];
}

// Segment table from the tensor table: thread s describes segment s.
__global__ void ss_segments_kernel(const SsTensor* __restrict__ tensors, int n, SsSegment* __restrict__ segs, int64_t nseg,
                                   int cpl, int out_bytes_per_piece) {
  int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= nseg) return;
  int lo = 0, hi = n;  // tensors[lo].seg_begin <= s < tensors[hi].seg_begin (hi == n: end)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (tensors[mid].seg_begin <= s) lo = mid; else hi = mid;
  }
  const SsTensor t = tensors[lo];
  SsSegment d;
  constexpr int64_t ITEMS = (int64_t)kSsSegWgs * kSsLanes;  // pieces, or 16-byte scale chunks, per segment
  if (s < t.seg_scale) {
    int64_t j = s - t.seg_begin;
    int64_t pieces = t.nblocks * (32 / cpl) - j * ITEMS;
    d.in = static_cast<const char*>(t.codes_h) + j * ITEMS * cpl;
    d.out = static_cast<char*>(t.codes_l) + j * ITEMS * out_bytes_per_piece;
    d.count = pieces < ITEMS ? pieces : ITEMS;
    d.kind = 0;
  } else {
    int64_t j = s - t.seg_scale;
    int64_t bytes = t.nblocks - j * ITEMS * 16;
    d.in = t.scales_h + j * ITEMS * 16;
    d.out = t.scales_l + j * ITEMS * 16;
    d.count = bytes < ITEMS * 16 ? bytes : ITEMS * 16;
    d.kind = 1;
  }
  segs[s] = d;
}

// ---- host side -----------------------------------------------------------------------------
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

template <int ANCHOR, int TARGET, bool HW>
static mx_status_t launch_ss(const SsTensor& t, int tie, hipStream_t stream) {
  constexpr int CPL = Piece<TARGET>::cpl;
  int64_t cw = ceil_div(t.nblocks * (32 / CPL), kSsLanes), sw = ceil_div(ceil_div(t.nblocks, 16), kSsLanes);
  if (cw + sw == 0) return MX_OK;
  if (cw + sw > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ss_kernel<ANCHOR, TARGET, HW>), dim3((unsigned)(cw + sw)), dim3(kSsLanes), 0, stream, t.codes_h,
                     t.scales_h, t.codes_l, t.scales_l, t.nblocks, cw, tie);
  return hipGetLastError() == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

template <int ANCHOR, int TARGET, bool HW>
static mx_status_t launch_ss_batched(const SsSegment* segs, int64_t nseg, int tie, hipStream_t stream) {
  hipLaunchKernelGGL((ss_batched_kernel<ANCHOR, TARGET, HW>), dim3((unsigned)(nseg * kSsSegWgs)), dim3(kSsLanes), 0, stream,
                     segs, tie);
  return hipGetLastError() == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

// Dispatch on (anchor, target, hw path) -> instantiated launcher.
template <typename F>
static mx_status_t ss_dispatch(int anchor, int target, bool hw, F&& f) {
#define MX_SS_CASE(A, T)                                              \
  if (anchor == A && target == T) {                                   \
    if (hw && Elem<T>::hw != HW_NONE) return f.template operator()<A, T, true>(); \
    return f.template operator()<A, T, false>();                      \
  }
  MX_SS_CASE(MX_INT8, MX_INT7)
  MX_SS_CASE(MX_INT8, MX_INT6)
  MX_SS_CASE(MX_INT8, MX_INT5)
  MX_SS_CASE(MX_INT8, MX_INT4)
  MX_SS_CASE(MX_INT8, MX_INT3)
  MX_SS_CASE(MX_INT8, MX_INT2)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP7_E3M3)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP6_E3M2)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP6_E2M3)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP5_E2M2)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP4_E2M1)
#undef MX_SS_CASE
  return MX_ERR_UNSUPPORTED;
}

struct SsOne {
  const SsTensor& t; int tie; hipStream_t stream;
  template <int A, int T, bool HW> mx_status_t operator()() const { return launch_ss<A, T, HW>(t, tie, stream); }
};
struct SsMany {
  const SsSegment* segs; int64_t nseg; int tie; hipStream_t stream;
  template <int A, int T, bool HW> mx_status_t operator()() const { return launch_ss_batched<A, T, HW>(segs, nseg, tie, stream); }
};

mx_status_t ss_launch_one(int anchor, int target, bool hw, const SsTensor& t, int tie, hipStream_t stream) {
  return ss_dispatch(anchor, target, hw, SsOne{t, tie, stream});
}

static inline int ss_cpl(int target_bits) { return target_bits % 2 == 0 ? 16 : 32; }

// Segments a tensor of nblocks blocks needs: code segments, scale segments.
static inline void ss_segments_of(int64_t nblocks, int cpl, int64_t* code_segs, int64_t* scale_segs) {
  const int64_t items = (int64_t)kSsSegWgs * kSsLanes;
  *code_segs = ceil_div(nblocks * (32 / cpl), items);
  *scale_segs = ceil_div(ceil_div(nblocks, 16), items);
}

size_t ss_workspace_bytes(int n, int64_t total_blocks) {
  // bound over both piece sizes: every tensor rounds up by at most one code and one scale segment
  const int64_t items = (int64_t)kSsSegWgs * kSsLanes;
  int64_t segs = total_blocks * 2 / items + total_blocks / (16 * items) + 2 * (int64_t)n + 2;
  return sizeof(SsTensor) * (size_t)n + sizeof(SsSegment) * (size_t)segs;
}

mx_status_t ss_launch_many(int anchor, int target, int target_bits, bool hw, int n, const SsTensor* h_tensors,
                           void* workspace, size_t workspace_bytes, int tie, hipStream_t stream) {
  const int cpl = ss_cpl(target_bits);
  // pass 1 on the host: segment ranges; nothing is launched before the sizes are known to fit
  int64_t nseg = 0;
  for (int i = 0; i < n; ++i) {
    int64_t cs, ss;
    ss_segments_of(h_tensors[i].nblocks, cpl, &cs, &ss);
    nseg += cs + ss;
  }
  if (nseg == 0) return MX_OK;
  if (nseg * kSsSegWgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  size_t tb = sizeof(SsTensor) * (size_t)n;
  if (workspace_bytes < tb + sizeof(SsSegment) * (size_t)nseg) return MX_ERR_WORKSPACE;
  SsTensor* table = static_cast<SsTensor*>(workspace);
  SsSegment* segs = reinterpret_cast<SsSegment*>(static_cast<char*>(workspace) + tb);
  int64_t acc = 0;
  SsTableChunk chunk;
  for (int base = 0; base < n; base += kSsTableChunk) {
    chunk.base = base;
    chunk.count = n - base < kSsTableChunk ? n - base : kSsTableChunk;
    for (int i = 0; i < chunk.count; ++i) {
      SsTensor t = h_tensors[base + i];
      int64_t cs, ss;
      ss_segments_of(t.nblocks, cpl, &cs, &ss);
      t.seg_begin = acc;
      t.seg_scale = acc + cs;
      acc += cs + ss;
      chunk.t[i] = t;
    }
    hipLaunchKernelGGL(ss_table_kernel, dim3(1), dim3(kSsTableChunk), 0, stream, chunk, table);
    if (hipGetLastError() != hipSuccess) return MX_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(ss_segments_kernel, dim3((unsigned)ceil_div(nseg, 256)), dim3(256), 0, stream, table, n, segs, nseg, cpl,
                     cpl * target_bits / 8);
  if (hipGetLastError() != hipSuccess) return MX_ERR_LAUNCH;
  return ss_dispatch(anchor, target, hw, SsMany{segs, nseg, tie, stream});
}

}  // namespace mx
