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

#include <atomic>

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

// Results are written once and not read again by this launch: non-temporal stores (measured: one to
// five points of HBM bandwidth, depending on the launch shape).
// Every pointer of a launch is device global memory, but one that a workgroup has loaded from a
// descriptor table carries no address space, and the compiler would reach through it with flat
// instructions (which also occupy the LDS path).  All accesses below therefore go through
// pointers cast to the global address space.
#define MX_GLOBAL __attribute__((address_space(1)))
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef u32x3 __attribute__((aligned(4))) u32x3_a4;

template <int W>
__device__ __forceinline__ void store_global(void* base, int64_t dword, const uint32_t (&v)[W]) {
  MX_GLOBAL uint32_t* p = (MX_GLOBAL uint32_t*)base + dword;
  if constexpr (W % 4 == 0) {
#pragma unroll
    for (int i = 0; i < W / 4; ++i)
      __builtin_nontemporal_store(u32x4{v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]}, (MX_GLOBAL u32x4*)p + i);
  } else if constexpr (W % 2 == 0) {
#pragma unroll
    for (int i = 0; i < W / 2; ++i) __builtin_nontemporal_store(u32x2{v[2 * i], v[2 * i + 1]}, (MX_GLOBAL u32x2*)p + i);
  } else if constexpr (W == 3) {
    *(MX_GLOBAL u32x3_a4*)p = u32x3{v[0], v[1], v[2]};   // one 96-bit store (needs only dword alignment)
  } else {
#pragma unroll
    for (int i = 0; i < W; ++i) p[i] = v[i];
  }
}

// codes per lane: half a block when every target width ends on a dword boundary there, else a whole block
template <int... TARGETS>
struct Piece { static constexpr int cpl = (((Elem<TARGETS>::bits % 2 == 0) && ...)) ? 16 : 32; };

// ---- the 64 pieces [p0, p0 + 64) of a run of `count` pieces, one per lane: load once, convert and
// store for every target of the launch.  A 6-bit target gives 12 bytes per lane; 96-bit stores cost
// about four points of HBM bandwidth against 128-bit ones (measured), so a wave that is all inside
// the run regroups its 192 result dwords through LDS and stores them 16 bytes per lane from 48 lanes.
template <int ANCHOR, bool HW, int... TARGETS>
__device__ __forceinline__ void ss_pieces(const void* __restrict__ in, void* const (&out)[kSsMaxTargets], int64_t p0, int64_t count,
                                          int tie) {
  constexpr int CPL = Piece<TARGETS...>::cpl, NIN = CPL / 4;
  constexpr int NSTAGED = ((CPL * Elem<TARGETS>::bits / 32 == 3 ? 1 : 0) + ...);
  __shared__ uint32_t stage[NSTAGED > 0 ? NSTAGED : 1][kSsLanes * 3];
  const int lane = threadIdx.x;
  const int64_t p = p0 + lane;
  const bool whole = p0 + kSsLanes <= count;   // the same for every lane of the wave
  if (!whole && p >= count) return;
  uint32_t x[NIN];
  const MX_GLOBAL u32x4* src = (const MX_GLOBAL u32x4*)in + p * (NIN / 4);
#pragma unroll
  for (int i = 0; i < NIN / 4; ++i) {
    u32x4 t = __builtin_nontemporal_load(src + i);
    x[4 * i] = t.x; x[4 * i + 1] = t.y; x[4 * i + 2] = t.z; x[4 * i + 3] = t.w;
  }
  int slot = 0, staged = 0;
  ([&] {
    constexpr int NOUT = CPL * Elem<TARGETS>::bits / 32;
    uint32_t y[NOUT];
    slice_piece<ANCHOR, TARGETS, HW && Elem<TARGETS>::hw != HW_NONE, CPL>(x, y, tie);
    if constexpr (NOUT == 3) {
      if (whole) {
        uint32_t* st = stage[staged];
        st[lane * 3] = y[0]; st[lane * 3 + 1] = y[1]; st[lane * 3 + 2] = y[2];
        __syncthreads();   // one wave per workgroup: orders the LDS writes before the reads below
        if (lane < 48) {
          u32x4 v = *reinterpret_cast<const u32x4*>(st + lane * 4);
          __builtin_nontemporal_store(v, (MX_GLOBAL u32x4*)((MX_GLOBAL uint32_t*)out[slot] + p0 * 3) + lane);
        }
      } else {
        store_global<NOUT>(out[slot], p * NOUT, y);
      }
      ++staged;
    } else {
      store_global<NOUT>(out[slot], p * NOUT, y);
    }
    ++slot;
  }(), ...);
}

// ---- 16 scale bytes per lane, for every target
template <int ANCHOR, int... TARGETS>
__device__ __forceinline__ void ss_scale_chunk(const uint8_t* __restrict__ sh, void* const (&out)[kSsMaxTargets], int64_t chunk,
                                               int64_t nbytes) {
  int64_t i0 = chunk * 16;
  if (i0 + 16 <= nbytes) {
    u32x4 v = *(const MX_GLOBAL u32x4*)(sh + i0);
    int slot = 0;
    ([&] {
      constexpr uint32_t DE = Elem<ANCHOR>::emax - Elem<TARGETS>::emax;
      u32x4 r = {scale_add_x4(v.x, DE), scale_add_x4(v.y, DE), scale_add_x4(v.z, DE), scale_add_x4(v.w, DE)};
      *(MX_GLOBAL u32x4*)((MX_GLOBAL uint8_t*)out[slot] + i0) = r;
      ++slot;
    }(), ...);
  } else {
    for (int64_t i = i0; i < nbytes; ++i) {
      uint32_t b = ((const MX_GLOBAL uint8_t*)sh)[i];
      int slot = 0;
      ([&] {
        constexpr uint32_t DE = Elem<ANCHOR>::emax - Elem<TARGETS>::emax;
        ((MX_GLOBAL uint8_t*)out[slot])[i] = (uint8_t)(b == 255u ? 255u : (b + DE > 254u ? 254u : b + DE));
        ++slot;
      }(), ...);
    }
  }
}

// kernel-argument form of one tensor (the flat launch needs no table)
struct SsFlatArgs {
  const void* codes_h;
  const uint8_t* scales_h;
  void* codes_l[kSsMaxTargets];
  void* scales_l[kSsMaxTargets];
  int64_t nblocks;    // scale bytes
  int64_t npieces;    // nblocks * block / CPL
  int64_t code_wgs;
};

// ---- one tensor: workgroups [0, code_wgs) convert pieces, the rest scale bytes
template <int ANCHOR, bool HW, int... TARGETS>
__global__ __launch_bounds__(kSsLanes) void ss_kernel(SsFlatArgs a, int tie) {
  int64_t wg = blockIdx.x;
  if (wg < a.code_wgs) {
    ss_pieces<ANCHOR, HW, TARGETS...>(a.codes_h, a.codes_l, wg * kSsLanes, a.npieces, tie);
  } else {
    int64_t c = (wg - a.code_wgs) * kSsLanes + threadIdx.x;
    if (c * 16 < a.nblocks) ss_scale_chunk<ANCHOR, TARGETS...>(a.scales_h, a.scales_l, c, a.nblocks);
  }
}

// ---- many tensors in one launch.  The work is cut into segments of 2^seg_shift workgroups, so a
// workgroup finds its segment with a shift and needs ONE dependent scalar load (the 64-byte
// segment descriptor) before its data load.  A descriptor that has to come from HBM while the
// memory system is saturated costs several points of bandwidth (measured: 77 % against 84 % of
// peak), so the first 8 workgroups of a segment - one per XCD, workgroups go round the XCDs -
// pull the descriptor `ahead` segments further on into their L2 with a one-lane load.
template <int ANCHOR, bool HW, int... TARGETS>
__global__ __launch_bounds__(kSsLanes) void ss_batched_kernel(const SsSegment* __restrict__ segs, int nseg, int seg_shift,
                                                              int ahead, int tie) {
  const int seg = blockIdx.x >> seg_shift, w = blockIdx.x & ((1 << seg_shift) - 1);
  const SsSegment s = segs[seg];
  int64_t item = (int64_t)w * kSsLanes + threadIdx.x;
  uint32_t warm = 0;
  if (w < 8 && threadIdx.x == 0) {
    int f = seg + ahead < nseg ? seg + ahead : nseg - 1;
    warm = *reinterpret_cast<const MX_GLOBAL uint32_t*>((const MX_GLOBAL SsSegment*)segs + f);
  }
  if (s.kind == 0) {
    ss_pieces<ANCHOR, HW, TARGETS...>(s.in, s.out, (int64_t)w * kSsLanes, s.count, tie);
  } else {
    if (item * 16 < s.count) ss_scale_chunk<ANCHOR, TARGETS...>(static_cast<const uint8_t*>(s.in), s.out, item, s.count);
  }
  asm volatile("" ::"v"(warm));  // keeps the load above alive; nothing waits for it before the wave's last instruction
}

struct SsPieceBytes { int out[kSsMaxTargets]; int n; int cpl; };

// Segment table of one chunk of tensors: thread j describes segment seg0 + j.
__global__ void ss_segments_kernel(SsChunk c, SsSegment* __restrict__ segs, int nseg_chunk, SsPieceBytes pb, int seg_shift,
                                   int block) {
  int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= nseg_chunk) return;
  const int stride = 4 + 2 * c.n_targets;
  int lo = 0, hi = c.count;  // first code segment of tensor lo <= s < that of tensor hi (hi == count: end)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if ((int)(uint32_t)c.w[mid * stride + 3] <= s) lo = mid; else hi = mid;
  }
  const int64_t* t = c.w + lo * stride;
  const int seg_begin = (int)(uint32_t)t[3], seg_scale = (int)(t[3] >> 32);
  const int64_t nblocks = t[2];
  const int64_t ITEMS = (int64_t)kSsLanes << seg_shift;  // pieces, or 16-byte scale chunks, per segment
  SsSegment d;
  d.pad = 0; d.pad2[0] = d.pad2[1] = 0;
  if (s < seg_scale) {
    int64_t j = s - seg_begin;
    int64_t pieces = nblocks * block / pb.cpl - j * ITEMS;
    d.in = reinterpret_cast<const char*>(t[0]) + j * ITEMS * pb.cpl;
    for (int q = 0; q < kSsMaxTargets; ++q)
      d.out[q] = q < pb.n ? reinterpret_cast<char*>(t[4 + q]) + j * ITEMS * pb.out[q] : nullptr;
    d.count = pieces < ITEMS ? pieces : ITEMS;
    d.kind = 0;
  } else {
    int64_t j = s - seg_scale;
    int64_t bytes = nblocks - j * ITEMS * 16;
    d.in = reinterpret_cast<const char*>(t[1]) + j * ITEMS * 16;
    for (int q = 0; q < kSsMaxTargets; ++q)
      d.out[q] = q < pb.n ? reinterpret_cast<char*>(t[4 + pb.n + q]) + j * ITEMS * 16 : nullptr;
    d.count = bytes < ITEMS * 16 ? bytes : ITEMS * 16;
    d.kind = 1;
  }
  segs[c.seg0 + s] = d;
}

// ---- host side -----------------------------------------------------------------------------
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

static inline int ss_cpl(const SsTargets& tg) {
  for (int q = 0; q < tg.n; ++q)
    if (tg.bits[q] % 2) return 32;
  return 16;
}

template <int ANCHOR, bool HW, int... TARGETS>
static mx_status_t launch_ss(const SsTensor& t, int block, int tie, hipStream_t stream) {
  constexpr int CPL = Piece<TARGETS...>::cpl;
  if ((t.nblocks * block) % CPL) return MX_ERR_UNSUPPORTED;   // odd widths convert whole runs of 32 codes
  const int64_t npieces = t.nblocks * block / CPL;
  int64_t cw = ceil_div(npieces, kSsLanes), sw = ceil_div(ceil_div(t.nblocks, 16), kSsLanes);
  if (cw + sw == 0) return MX_OK;
  if (cw + sw > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  SsFlatArgs a;
  a.codes_h = t.codes_h; a.scales_h = t.scales_h; a.nblocks = t.nblocks; a.npieces = npieces; a.code_wgs = cw;
  for (int q = 0; q < kSsMaxTargets; ++q) { a.codes_l[q] = t.codes_l[q]; a.scales_l[q] = t.scales_l[q]; }
  hipLaunchKernelGGL((ss_kernel<ANCHOR, HW, TARGETS...>), dim3((unsigned)(cw + sw)), dim3(kSsLanes), 0, stream, a, tie);
  return launch_status("a Slice-and-Scale kernel");
}

template <int ANCHOR, bool HW, int... TARGETS>
static mx_status_t launch_ss_batched(const SsSegment* segs, int64_t nseg, int seg_shift, int tie, hipStream_t stream) {
  // descriptors are pulled in about 2048 .. 8192 workgroups ahead of their first use (measured optimum)
  const int ahead = seg_shift >= kSsSegShiftLarge ? 2 : 64;
  // With three targets the launch writes twice what it reads, and HBM then does better with fewer waves in
  // flight (a narrower front of open pages): unused dynamic LDS holds a CU at about 22 workgroups (measured:
  // 69.9 -> 72.3 % of peak; every launch with fewer targets loses bandwidth under any such cap).
  constexpr unsigned occupancy_pad = sizeof...(TARGETS) >= 3 ? 5632 : 0;
  hipLaunchKernelGGL((ss_batched_kernel<ANCHOR, HW, TARGETS...>), dim3((unsigned)(nseg << seg_shift)), dim3(kSsLanes), occupancy_pad, stream,
                     segs, (int)nseg, seg_shift, ahead, tie);
  return launch_status("a Slice-and-Scale kernel");
}

// Dispatch on (anchor, target list, hw path) -> instantiated launcher.  Single targets: every narrower format of
// the family.  Several targets in one pass (the anchor is read once): the benchmark's "every lower format" sets.
template <typename F>
static mx_status_t ss_dispatch(int anchor, const SsTargets& tg, bool hw, F&& f) {
  const int t0 = tg.elem[0], t1 = tg.n > 1 ? tg.elem[1] : -1, t2 = tg.n > 2 ? tg.elem[2] : -1;
#define MX_SS_CASE(A, ...)                                                   \
  {                                                                          \
    constexpr int want[] = {__VA_ARGS__, -1, -1};                            \
    if (anchor == A && t0 == want[0] && t1 == want[1] && t2 == want[2]) {    \
      if (hw) return f.template operator()<A, true, __VA_ARGS__>();          \
      return f.template operator()<A, false, __VA_ARGS__>();                 \
    }                                                                        \
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
  MX_SS_CASE(MX_INT8, MX_INT6, MX_INT4)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP6_E3M2, MX_FP6_E2M3, MX_FP4_E2M1)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP6_E3M2, MX_FP4_E2M1)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP6_E2M3, MX_FP4_E2M1)
  MX_SS_CASE(MX_FP8_E4M3, MX_FP6_E3M2, MX_FP6_E2M3)
#undef MX_SS_CASE
  return MX_ERR_UNSUPPORTED;
}

struct SsOne {
  const SsTensor& t; int block; int tie; hipStream_t stream;
  template <int A, bool HW, int... T> mx_status_t operator()() const { return launch_ss<A, HW, T...>(t, block, tie, stream); }
};
struct SsMany {
  const SsSegment* segs; int64_t nseg; int seg_shift; int tie; hipStream_t stream;
  template <int A, bool HW, int... T> mx_status_t operator()() const {
    return launch_ss_batched<A, HW, T...>(segs, nseg, seg_shift, tie, stream);
  }
};

struct SsProbe {   // "is there a kernel for this target list?" without launching anything
  template <int A, bool HW, int... T> mx_status_t operator()() const { return MX_OK; }
};

mx_status_t ss_launch_one(int anchor, const SsTargets& tg, bool hw, const SsTensor& t, int block, int tie, hipStream_t stream) {
  return ss_dispatch(anchor, tg, hw, SsOne{t, block, tie, stream});
}

// Segments a tensor of nblocks blocks needs: code segments, scale segments.
static inline void ss_segments_of(int64_t nblocks, int block, int cpl, int seg_shift, int64_t* code_segs, int64_t* scale_segs) {
  const int64_t items = (int64_t)kSsLanes << seg_shift;
  *code_segs = ceil_div(nblocks * block / cpl, items);
  *scale_segs = ceil_div(ceil_div(nblocks, 16), items);
}

static int64_t ss_count_segments(const SsBatch& batch, int block, int cpl, int seg_shift) {
  int64_t nseg = 0;
  for (int i = 0; i < batch.n; ++i) {
    int64_t cs, ss;
    ss_segments_of(batch.anchors[i].outer * batch.anchors[i].nblocks, block, cpl, seg_shift, &cs, &ss);
    nseg += cs + ss;
  }
  return nseg;
}

size_t ss_workspace_bytes(int n, int64_t total_blocks) {
  // bound over every block size (up to 128: 8 pieces of 16 codes per block), both piece sizes and both segment
  // sizes: every tensor rounds up by at most one code and one scale segment, and small segments need the most
  // descriptors
  const int64_t items = (int64_t)kSsLanes << kSsSegShiftSmall;
  int64_t segs = total_blocks * 8 / items + total_blocks / (16 * items) + 2 * (int64_t)n + 2;
  return sizeof(SsSegment) * (size_t)segs;
}

mx_status_t ss_launch_many(int anchor, const SsTargets& tg, bool hw, const SsBatch& batch, int block, void* workspace,
                           size_t workspace_bytes, int tie, hipStream_t stream) {
  const int cpl = ss_cpl(tg), n = batch.n;
  for (int i = 0; i < n; ++i)
    if ((batch.anchors[i].outer * batch.anchors[i].nblocks * block) % cpl) return MX_ERR_UNSUPPORTED;   // odd widths convert whole runs of 32 codes
  // pass 1 on the host: segment ranges; nothing is launched before the sizes are known to fit.  Large segments
  // unless their padding (workgroups that find nothing to do) would exceed 1/32 of the launch.
  int seg_shift = kSsSegShiftLarge;
  int64_t nseg = ss_count_segments(batch, block, cpl, seg_shift);
  {
    int64_t small = ss_count_segments(batch, block, cpl, kSsSegShiftSmall);
    if ((nseg << kSsSegShiftLarge) - (small << kSsSegShiftSmall) > (small << kSsSegShiftSmall) / 32) {
      seg_shift = kSsSegShiftSmall;
      nseg = small;
    }
  }
  if (nseg == 0) return MX_OK;
  if ((nseg << seg_shift) > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  if (workspace_bytes < sizeof(SsSegment) * (size_t)nseg) return MX_ERR_WORKSPACE;
  // an unsupported target list must fail before anything is launched
  {
    mx_status_t st = ss_dispatch(anchor, tg, hw, SsProbe{});
    if (st != MX_OK) return st;
  }
  SsSegment* segs = static_cast<SsSegment*>(workspace);
  SsPieceBytes pb;
  pb.n = tg.n; pb.cpl = cpl;
  for (int q = 0; q < kSsMaxTargets; ++q) pb.out[q] = q < tg.n ? cpl * tg.bits[q] / 8 : 0;
  // the segment table, written by one small launch per chunk of tensors
  const int stride = 4 + 2 * tg.n, cap = kSsChunkWords / stride;
  int64_t seg0 = 0;
  SsChunk chunk;
  for (int base = 0; base < n; base += cap) {
    chunk.count = n - base < cap ? n - base : cap;
    chunk.n_targets = tg.n;
    chunk.seg0 = seg0;
    int64_t acc = 0;
    for (int i = 0; i < chunk.count; ++i) {
      const SsTensor t = batch.tensor(base + i);
      int64_t cs, ss;
      ss_segments_of(t.nblocks, block, cpl, seg_shift, &cs, &ss);
      int64_t* w = chunk.w + i * stride;
      w[0] = (int64_t)(uintptr_t)t.codes_h;
      w[1] = (int64_t)(uintptr_t)t.scales_h;
      w[2] = t.nblocks;
      w[3] = acc | ((acc + cs) << 32);
      for (int q = 0; q < tg.n; ++q) {
        w[4 + q] = (int64_t)(uintptr_t)t.codes_l[q];
        w[4 + tg.n + q] = (int64_t)(uintptr_t)t.scales_l[q];
      }
      acc += cs + ss;
    }
    if (acc > 0) {
      hipLaunchKernelGGL(ss_segments_kernel, dim3((unsigned)ceil_div(acc, 256)), dim3(256), 0, stream, chunk, segs, (int)acc, pb,
                         seg_shift, block);
      if (launch_status("the segment table writer") != MX_OK) return MX_ERR_LAUNCH;
    }
    seg0 += acc;
  }
  return ss_dispatch(anchor, tg, hw, SsMany{segs, nseg, seg_shift, tie, stream});
}

// ---- a segment table that lives in the library, for callers that cannot allocate or lend device memory
// `scratch` is a file-scope device array: every GPU the library runs on holds its own copy, at its own address, until
// the process ends.  In host code the array's name is only a handle for the runtime, never an address to pass to a
// kernel: the address on the current device comes from hipGetSymbolAddress, is asked for once per device and kept.
static_assert(sizeof(SsSegment) == 64 && kSsStaticSegments == MX_SS_NOALLOC_MAX_SEGMENTS, "the size mx.h states");
static __device__ __align__(256) unsigned char scratch[kSsStaticSegments * sizeof(SsSegment)];

mx_status_t ss_static_workspace(void** ptr, size_t* bytes) {
  static std::atomic<void*> address[64];   // per device; a second thread asking at the same time gets the same answer
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MX_ERR_LAUNCH;
  void* p = address[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return MX_ERR_LAUNCH;
    }
    address[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  *bytes = sizeof(scratch);
  return MX_OK;
}

}  // namespace mx
