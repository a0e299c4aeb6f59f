// Slice-and-Scale kernels (Eq. (4) SSMXINT, Eq. (6) SSMXFP): 8-bit anchor -> narrower target.
//
// The packed layout is a flat run of blocks, so the conversion is a streaming map with no
// reduction and no neighbour dependence: one lane converts one block (32 anchor bytes in two
// 128-bit loads -> `bits` dwords out), and the scale bytes are a second, independent stream
// (byte + De, saturating) handled by workgroups of their own at 16 bytes per lane.
#include "mx_device.h"
#include "mx_launch.h"

namespace mx {

// ---- one block: 32 anchor codes (8 dwords) -> W = target bits dwords
template <int ANCHOR, int TARGET, bool HW>
__device__ __forceinline__ void slice_block(const uint32_t (&in)[8], uint32_t (&out)[Elem<TARGET>::bits], int tie) {
  using T = Elem<TARGET>;
  if constexpr (Elem<ANCHOR>::is_int) {
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = slice_int8x4<T::bits>(in[i], tie);
    pack_block_bytes<T::bits>(c, out);
  } else {
    constexpr int DE = Elem<ANCHOR>::emax - T::emax;
    const float two_de = __uint_as_float((uint32_t)(127 + DE) << 23);
    if constexpr (HW && T::hw == HW_FP4) {
      // E4M3 -> fp32 (exact) -> E2M1 with the 2^De division folded into the conversion's scale
#pragma unroll
      for (int j = 0; j < 4; ++j) {
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
      // E4M3 -> fp16 (exact: 4 significant bits, exponents -9..8) -> 32 FP6 codes in one instruction
      f16x32 h;
      const float one = __uint_as_float(127u << 23);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint32_t x = e4m3_nan_to_max(in[i]);
        f16x2 a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(x, one, false);
        f16x2 b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(x, one, true);
        h[4 * i] = a.x; h[4 * i + 1] = a.y; h[4 * i + 2] = b.x; h[4 * i + 3] = b.y;
      }
      u32x6 p = cvt_pk32_fp6_f16<T::hw == HW_BF6>(h, two_de);
#pragma unroll
      for (int i = 0; i < 6; ++i) out[i] = p[i];
    } else {
      uint32_t c[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint32_t x = e4m3_nan_to_max(in[i]);
        uint32_t r = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) r |= slice_e4m3_sw<TARGET>((x >> (8 * b)) & 0xFFu, tie) << (8 * b);
        c[i] = r;
      }
      pack_block_bytes<T::bits>(c, out);
    }
  }
}

// ---- the work of one workgroup on one tensor
// Code workgroups: lane l of workgroup g converts blocks g*256*U + l + 256*u, u < U.
template <int ANCHOR, int TARGET, bool HW, int U>
__device__ __forceinline__ void ss_codes_tile(const uint32_t* __restrict__ ch, uint32_t* __restrict__ cl, int64_t nblocks,
                                              int64_t wg, int tie) {
  constexpr int W = Elem<TARGET>::bits;
  int64_t b0 = wg * (256 * U) + threadIdx.x;
  uint32_t in[U][8];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t b = b0 + 256 * u;
    if (b < nblocks) {
      const u32x4* p = reinterpret_cast<const u32x4*>(ch + b * 8);
      u32x4 lo = __builtin_nontemporal_load(p), hi = __builtin_nontemporal_load(p + 1);
      in[u][0] = lo.x; in[u][1] = lo.y; in[u][2] = lo.z; in[u][3] = lo.w;
      in[u][4] = hi.x; in[u][5] = hi.y; in[u][6] = hi.z; in[u][7] = hi.w;
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t b = b0 + 256 * u;
    if (b < nblocks) {
      uint32_t out[W];
      slice_block<ANCHOR, TARGET, HW>(in[u], out, tie);
      store_dwords<W>(cl + b * W, out);
    }
  }
}

// Scale workgroups: lane l of workgroup g updates scale bytes [16*(g*256+l), +16).
template <int DE>
__device__ __forceinline__ void ss_scales_tile(const uint8_t* __restrict__ sh, uint8_t* __restrict__ sl, int64_t nblocks,
                                               int64_t wg) {
  int64_t i0 = (wg * 256 + threadIdx.x) * 16;
  if (i0 + 16 <= nblocks) {
    u32x4 v = *reinterpret_cast<const u32x4*>(sh + i0);
    v.x = scale_add_x4(v.x, DE); v.y = scale_add_x4(v.y, DE); v.z = scale_add_x4(v.z, DE); v.w = scale_add_x4(v.w, DE);
    *reinterpret_cast<u32x4*>(sl + i0) = v;
  } else {
    for (int64_t i = i0; i < nblocks; ++i) {
      uint32_t b = sh[i];
      uint32_t r = b == 255u ? 255u : (b + DE > 254u ? 254u : b + DE);
      sl[i] = (uint8_t)r;
    }
  }
}

template <int ANCHOR, int TARGET, bool HW, int U>
__global__ __launch_bounds__(256) void ss_kernel(const uint32_t* __restrict__ ch, const uint8_t* __restrict__ sh,
                                                 uint32_t* __restrict__ cl, uint8_t* __restrict__ sl, int64_t nblocks,
                                                 int64_t code_wgs, int tie) {
  constexpr int DE = Elem<ANCHOR>::emax - Elem<TARGET>::emax;
  int64_t wg = blockIdx.x;
  if (wg < code_wgs) ss_codes_tile<ANCHOR, TARGET, HW, U>(ch, cl, nblocks, wg, tie);
  else ss_scales_tile<DE>(sh, sl, nblocks, wg - code_wgs);
}

// Batched form: tensor i owns workgroups [wg_begin, next tensor's wg_begin): first its code
// workgroups, from wg_scale on its scale workgroups.  The table lives in caller-provided device
// memory and is written there by ss_table_kernel from kernel arguments (no host buffer has to
// outlive the call, nothing is copied).
template <int ANCHOR, int TARGET, bool HW, int U>
__global__ __launch_bounds__(256) void ss_batched_kernel(const SsTensor* __restrict__ tensors, int n, int tie) {
  constexpr int DE = Elem<ANCHOR>::emax - Elem<TARGET>::emax;
  int64_t wg = blockIdx.x;
  int lo = 0, hi = n;  // invariant: tensors[lo].wg_begin <= wg, and wg < tensors[hi].wg_begin if hi < n
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (tensors[mid].wg_begin <= wg) lo = mid; else hi = mid;
  }
  lo = __builtin_amdgcn_readfirstlane(lo);
  const SsTensor t = tensors[lo];
  if (wg < t.wg_scale)
    ss_codes_tile<ANCHOR, TARGET, HW, U>(reinterpret_cast<const uint32_t*>(t.codes_h), reinterpret_cast<uint32_t*>(t.codes_l),
                                         t.nblocks, wg - t.wg_begin, tie);
  else
    ss_scales_tile<DE>(t.scales_h, t.scales_l, t.nblocks, wg - t.wg_scale);
}

__global__ void ss_table_kernel(SsTableChunk chunk, SsTensor* __restrict__ table) {
  int i = threadIdx.x;
  if (i < chunk.count) table[chunk.base + i] = chunk.t[i];
}

// ---- host side -----------------------------------------------------------------------------
constexpr int kSsUnroll = 4;

static inline int64_t ss_code_wgs(int64_t nblocks) { return (nblocks + 256 * kSsUnroll - 1) / (256 * kSsUnroll); }
static inline int64_t ss_scale_wgs(int64_t nblocks) { return (nblocks + 4095) / 4096; }

template <int ANCHOR, int TARGET, bool HW>
static mx_status_t launch_ss(const SsTensor& t, int tie, hipStream_t stream) {
  int64_t cw = ss_code_wgs(t.nblocks), sw = ss_scale_wgs(t.nblocks);
  if (cw + sw == 0) return MX_OK;
  if (cw + sw > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((ss_kernel<ANCHOR, TARGET, HW, kSsUnroll>), dim3((unsigned)(cw + sw)), dim3(256), 0, stream,
                     reinterpret_cast<const uint32_t*>(t.codes_h), t.scales_h, reinterpret_cast<uint32_t*>(t.codes_l),
                     t.scales_l, t.nblocks, cw, tie);
  return hipGetLastError() == hipSuccess ? MX_OK : MX_ERR_LAUNCH;
}

template <int ANCHOR, int TARGET, bool HW>
static mx_status_t launch_ss_batched(const SsTensor* d_tensors, int n, int64_t total_wgs, int tie, hipStream_t stream) {
  hipLaunchKernelGGL((ss_batched_kernel<ANCHOR, TARGET, HW, kSsUnroll>), dim3((unsigned)total_wgs), dim3(256), 0, stream,
                     d_tensors, n, tie);
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
  const SsTensor* d_tensors; int n; int64_t total; int tie; hipStream_t stream;
  template <int A, int T, bool HW> mx_status_t operator()() const {
    return launch_ss_batched<A, T, HW>(d_tensors, n, total, tie, stream);
  }
};

mx_status_t ss_launch_one(int anchor, int target, bool hw, const SsTensor& t, int tie, hipStream_t stream) {
  return ss_dispatch(anchor, target, hw, SsOne{t, tie, stream});
}

mx_status_t ss_launch_many(int anchor, int target, bool hw, int n, const SsTensor* h_tensors, void* workspace,
                           int tie, hipStream_t stream) {
  SsTensor* table = static_cast<SsTensor*>(workspace);
  int64_t acc = 0;
  SsTableChunk chunk;
  for (int base = 0; base < n; base += kSsTableChunk) {
    chunk.base = base;
    chunk.count = n - base < kSsTableChunk ? n - base : kSsTableChunk;
    for (int i = 0; i < chunk.count; ++i) {
      SsTensor t = h_tensors[base + i];
      t.wg_begin = acc;
      acc += ss_code_wgs(t.nblocks);
      t.wg_scale = acc;
      acc += ss_scale_wgs(t.nblocks);
      chunk.t[i] = t;
    }
    if (acc > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;   // checked before the last (the only effective) launch
    hipLaunchKernelGGL(ss_table_kernel, dim3(1), dim3(kSsTableChunk), 0, stream, chunk, table);
    if (hipGetLastError() != hipSuccess) return MX_ERR_LAUNCH;
  }
  if (acc == 0) return MX_OK;
  return ss_dispatch(anchor, target, hw, SsMany{table, n, acc, tie, stream});
}

}  // namespace mx
