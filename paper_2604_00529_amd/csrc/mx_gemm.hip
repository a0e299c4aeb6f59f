// Fused consumer of an elastic-precision checkpoint (Sec. 3.5 "Inference": the model runs with
// W_t = Q_{A->t}(W_A) generated on demand): C = DQ(A) * DQ(SS(W_A -> MXFP4))^T, where A holds MXFP8
// (E4M3) activations and W_A is the stored MXFP8 (E4M3) anchor, both blocked by 32 along K.  The anchor
// is sliced to E2M1 in registers (Eq. (6)) and fed, with the E8M0 block scales (Eq. (6) scale step), to
// the CDNA4 scaled MFMA v_mfma_scale_f32_16x16x128_f8f6f4; accumulation is fp32.  W_t never exists in
// memory -- unless the caller lends a workspace: then, for large M, W_t is written there once per call and
// multiplied by a kernel without slicing waves (last part of this file), and shapes with few tiles of C
// split K over several workgroups whose partial sums pass through it.
//
// Kernels by shape: M <= 16 decode (streams W once), 16 < M <= 48 the same stream against two or three row
// tiles of A, M > 48 the LDS-tiled persistent kernel with producer and consumer waves.  Each of them also exists in a
// form for a W_t that the caller keeps (MXFP4 codes in memory, converted once per precision switch): 8-byte loads where
// 16 anchor bytes were loaded, no slicing and no scale step, the same instruction stream otherwise -- every output's
// sum over K runs in the same order in all kernels, so all ways through this file return the same bits (a K split
// aside).
//
// Operand layout of that instruction, established by one-hot probes on the GPU:
//   lane l = (i = l % 16, g = l / 16).  An FP4 operand lane holds the 32 codes of K-block g of row /
//   column i (k = 32 g + nibble).  An FP8 operand lane holds two 16-byte runs: k = 16 g + [0, 16) and
//   k = 64 + 16 g + [0, 16).  The scale byte of lane (i, g) applies to K-block g of row / column i, for
//   either operand type.  Result register j of lane l is C[4 (l / 16) + j][l % 16].
#include "mx_device.h"
#include "mx_launch.h"

#include <atomic>
#include <type_traits>

namespace mx {

typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int kDeltaE_E4M3_E2M1 = Elem<MX_FP8_E4M3>::emax - Elem<MX_FP4_E2M1>::emax;  // 6

constexpr int kMidmMaxM = 48;     // 16 < M <= 48: the streaming kernel with fragment loads for A (at M = 64 the tiled kernel is faster: 25 against 30 us)

// ------------------------------------------------------------------ M <= 16 (decode): coalesced loads, transposed in LDS
// With M <= 16 the kernel does little but stream W once.  Measured on the 58.7 MB anchor of the 4096 x 14336 layer: read
// with MFMA fragment loads (the 64 lanes of a load on 16 rows, 16 bytes each) the matrix alone takes 12.3 us, read with
// loads whose lanes take consecutive 16 bytes of one row 9.7 us.  So every load of W here is one contiguous 1 KB -- lane l
// takes bytes 16 l .. 16 l + 15 of a row's 1 KB K-chunk, half a block -- and the way into the operand layout goes through
// a wave-private LDS tile, the anchor sliced to E2M1 (Eq. (6)) on the way in.  One workgroup of 4 waves per 16 NT output
// columns; K is cut into chunks of 8 K-steps (a K-step is 128 elements = 4 blocks, one per lane group; a chunk is 1024
// elements) dealt round-robin to the waves, and the four partial sums are added in a fixed order through LDS
// (deterministic).
//
// The rows of a chunk pass through a ring of kDecodeRing register sets: a wave slices row r as soon as it has landed
// and only then requests row r + kDecodeRing.  (With all 16 NT loads of a chunk issued up front a wave sat behind its
// own load instructions -- the memory pipe takes them only as fast as it drains -- while rows it could have sliced had
// long arrived, and all the slicing piled up behind the stream: 15.7 us against 13.1 us for the 58.7 MB matrix.  Rings
// of 5 to 8 rows measure the same; 12 and more are slower again.)  The MFMAs of a column tile follow its sixteenth row.
//
// LDS tile of a wave, used twice per chunk.  First the A chunk, which goes straight from global memory into LDS (no
// registers in between) and from there into the wave's fragment registers: 16 rows of 64 slots of 16 bytes, rows padded
// by one slot so that the 16 lanes that read one slot of 16 consecutive rows hit 16 different bank groups.  Then, per
// column tile, 16 rows of 32 slots (one row = the 512 bytes of a column's sliced chunk) with slot s of row r at slot
// s ^ (r & 15), for the same reason; a row is still written as one contiguous (permuted) run.
constexpr int kDecodeARow = 1024 + 16;          // A rows are padded by one slot: row r, slot s -> bank group (r + s) % 16
constexpr int kDecodeTile = 16 * kDecodeARow;   // (>= the 8 KB of a sliced W tile)
constexpr int kDecodeRing = 6;                  // rows of W in flight per wave
constexpr int kDecodeRingSliced = 16;           // ... of a W_t kept by the caller (8-byte loads: the same bytes in flight and more; 6: 10.0 us, 16: 9.5 us per call at 16 x 14336 x 4096)
constexpr int decode_smem_bytes(int nt) { return 4 * kDecodeTile + 3 * nt * 4 * 64 * (int)sizeof(float); }

// 16 E4M3 anchor codes (4 dwords) -> 16 E2M1 codes (2 dwords): the Slice-and-Scale element step on half a block
__device__ __forceinline__ void slice_half_block_e2m1(const u32x4& in4, uint32_t (&out)[2]) {
  const float two_de = __uint_as_float((uint32_t)(127 + kDeltaE_E4M3_E2M1) << 23);
  const uint32_t in[4] = {in4.x, in4.y, in4.z, in4.w};
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    uint32_t w = 0;
    static_for<0, 2>([&](auto hh) {
      constexpr int H = decltype(hh)::value;
      uint32_t x = e4m3_nan_to_max(in[2 * j + H]);
      f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8(x, false);
      f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8(x, true);
      w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, a.x, a.y, two_de, 2 * H);
      w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, b.x, b.y, two_de, 2 * H + 1);
    });
    out[j] = w;
  }
}

// Raw buffer over `bytes` bytes at p (stride 0; the last word is the gfx9 descriptor default), and a 128-bit load at
// byte offset `lane_off` (a register) + `row_off` (a scalar); NT marks W, which is read once, as non-temporal.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buffer(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
template <bool NT>
__device__ __forceinline__ u32x4 buffer_load_x4(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off, uint32_t row_off) {
  auto v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_off, (int)row_off, NT ? 2 : 0);
  return u32x4{v[0], v[1], v[2], v[3]};
}

template <bool NT>
__device__ __forceinline__ u32x2 buffer_load_x2(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off, uint32_t row_off) {
  auto v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_off, (int)row_off, NT ? 2 : 0);
  return u32x2{v[0], v[1]};
}

// Byte g of each of the 8 dwords of a row's 32-byte scale chunk (the K-block that lane group g holds in each of the
// chunk's 8 K-steps): K-steps 0-3 packed into out[0], 4-7 into out[1].
__device__ __forceinline__ void pack_lane_scales(const u32x4& lo, const u32x4& hi, int g, uint32_t (&out)[2]) {
  const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  const int sh = 8 * g;
#pragma unroll
  for (int h = 0; h < 2; ++h)
    out[h] = ((w[4 * h] >> sh) & 0xFFu) | (((w[4 * h + 1] >> sh) & 0xFFu) << 8) | (((w[4 * h + 2] >> sh) & 0xFFu) << 16) |
             ((w[4 * h + 3] >> sh) << 24);
}

// s_waitcnt vmcnt(n) alone on gfx9: vmcnt is split over bits 3:0 and 15:14 of the immediate; the other counters stay at
// their maxima (expcnt 7 in bits 6:4, lgkmcnt 15 in bits 11:8)
constexpr int wait_vmcnt(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// Orders the LDS traffic of one wave for the compiler (the hardware executes a wave's LDS instructions in order, so
// what other lanes wrote is there when the read executes) without making it wait for the global loads in flight.
__device__ __forceinline__ void wave_lds_order() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_wave_barrier();
}


// NT column tiles of 16 per workgroup: 2, or 1 when that is what it takes to give every compute unit a workgroup.
// SLICED: W is a W_t the caller keeps (MXFP4 codes [N][K / 2], scale bytes already those of the target): lane l loads
// the 8 bytes it would otherwise have made of its 16 anchor codes, and the rest is the same instruction for instruction,
// so both forms of the kernel return the same bits.
template <int NT, bool SLICED>
__global__ __launch_bounds__(256, 2) void gemm_fp4_decode_kernel(const uint8_t* __restrict__ a_codes,
                                                                 const uint8_t* __restrict__ a_scales,
                                                                 const uint8_t* __restrict__ w_codes,
                                                                 const uint8_t* __restrict__ w_scales, float* __restrict__ c,
                                                                 int M, int N, int K, int64_t ldc) {
  constexpr int R = 16 * NT, D = SLICED ? kDecodeRingSliced : kDecodeRing;   // rows of W per chunk; rows in flight
  static_assert(D <= 16 && 8 * 1024 <= kDecodeTile, "the ring is refilled across column tiles; one 8 KB tile of sliced codes");
  extern __shared__ __attribute__((aligned(16))) uint8_t decode_smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 15, g = lane >> 4;
  const int KB = K / 32, ksteps = K / 128, chunks = (ksteps + 7) / 8;
  uint8_t* tile = decode_smem + wave * kDecodeTile;
  f32x4* red = reinterpret_cast<f32x4*>(decode_smem + 4 * kDecodeTile);   // [3][NT][64] partial sums of 4 outputs
  f32x4 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int col0 = blockIdx.x * NT * 16;
  // fragment-side view of the columns (lane (i, g) <-> column i of a tile): scale rows and the output
  int ncol[NT];   // columns past the edge are computed from column N - 1 and never stored
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) ncol[nt] = col0 + nt * 16 + i;
  // Buffer loads: the loads of a chunk share one offset register per operand (the row is a scalar offset).  The host
  // has checked that both matrices are smaller than 4 GiB.  Reads past the end of a buffer return zero.
  const __amdgpu_buffer_rsrc_t a_rsrc = make_buffer(a_codes, (uint32_t)M * (uint32_t)K);
  using WReg = std::conditional_t<SLICED, u32x2, u32x4>;                  // a lane's 16 codes of W as loaded
  constexpr uint32_t kWLane = SLICED ? 8u : 16u, kWChunk = SLICED ? 512u : 1024u;
  const uint32_t w_row = SLICED ? (uint32_t)K / 2u : (uint32_t)K;         // bytes per row of W
  const __amdgpu_buffer_rsrc_t w_rsrc = make_buffer(w_codes, (uint32_t)N * w_row);
  const __amdgpu_buffer_rsrc_t as_rsrc = make_buffer(a_scales, (uint32_t)M * (uint32_t)KB);
  const __amdgpu_buffer_rsrc_t ws_rsrc = make_buffer(w_scales, (uint32_t)N * (uint32_t)KB);
  for (int chunk = wave; chunk < chunks; chunk += 4) {
    // Lane l covers K-step l / 8 of the chunk.  In a ragged last chunk the lanes of K-steps that do not exist load the
    // chunk's first 16 bytes instead (every access stays inside the matrices); what they load is sliced like the rest
    // and multiplied with zero A fragments.  Rows of A past M read row M - 1; their products land in output rows that
    // are not stored.
    const int steps = ksteps - chunk * 8 < 8 ? ksteps - chunk * 8 : 8;
    const uint32_t lane_off = (lane >> 3) < steps ? 16u * (uint32_t)lane : 0u;
    const uint32_t chunk_off = (uint32_t)chunk * 1024u;
    const uint32_t w_lane_off = (lane >> 3) < steps ? kWLane * (uint32_t)lane : 0u;
    auto load_row = [&](int r) {   // row r of the chunk: column col0 + r, one contiguous 1 KB (512 bytes of a sliced W)
      const int n = col0 + r < N ? col0 + r : N - 1;
      if constexpr (SLICED) return buffer_load_x2<true>(w_rsrc, w_lane_off, (uint32_t)n * w_row + (uint32_t)chunk * kWChunk);
      else return buffer_load_x4<true>(w_rsrc, w_lane_off, (uint32_t)n * w_row + (uint32_t)chunk * kWChunk);
    };
    // A: the chunk of each row (1 KB, lane l <-> 16 bytes) goes straight from global memory into the wave's LDS tile, no
    // registers in between; the hardware puts lane l's 16 bytes at slot l of the row.  These loads are requested before
    // everything else and are the oldest in flight.
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const uint32_t row = r < M ? r : M - 1;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (__attribute__((address_space(3))) void*)(decode_smem + wave * kDecodeTile + r * kDecodeARow),
                                               16, (int)lane_off, (int)(row * (uint32_t)K + chunk_off), 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // The 32 scale bytes of the chunk per row / column.  In a ragged last chunk the 32 bytes run past the row's end: into
    // the next row, or past the end of the array, where a buffer load returns zeros; those bytes belong to K-steps that
    // do not exist and are replaced below.
    u32x4 aslo, ashi, wslo[NT], wshi[NT];
    {
      const uint32_t ao = (uint32_t)(i < M ? i : M - 1) * (uint32_t)KB + (uint32_t)chunk * 32u;
      aslo = buffer_load_x4<false>(as_rsrc, ao, 0u);
      ashi = buffer_load_x4<false>(as_rsrc, ao + 16u, 0u);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const uint32_t wo = (uint32_t)(ncol[nt] < N ? ncol[nt] : N - 1) * (uint32_t)KB + (uint32_t)chunk * 32u;
        wslo[nt] = buffer_load_x4<false>(ws_rsrc, wo, 0u);
        wshi[nt] = buffer_load_x4<false>(ws_rsrc, wo + 16u, 0u);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    WReg ring[D];
#pragma unroll
    for (int r = 0; r < D; ++r) ring[r] = load_row(r);
    __builtin_amdgcn_sched_barrier(0);
    // the first D rows of W have been requested after A and the scale bytes: once no more than D loads are outstanding,
    // A is in the tile and the scale bytes are in their registers
    __builtin_amdgcn_s_waitcnt(wait_vmcnt(D));
    wave_lds_order();
    // the 8 x 2 fragment runs of lane (i, g): slots 8 p + g and 8 p + 4 + g of row i; zeros for K-steps that do not exist
    i32x8 af[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      u32x4 t0 = *reinterpret_cast<const u32x4*>(tile + i * kDecodeARow + 16 * (8 * p + g));
      u32x4 t1 = *reinterpret_cast<const u32x4*>(tile + i * kDecodeARow + 16 * (8 * p + 4 + g));
      af[p] = i32x8{(int)t0.x, (int)t0.y, (int)t0.z, (int)t0.w, (int)t1.x, (int)t1.y, (int)t1.z, (int)t1.w};
      if (p >= steps) af[p] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    // the 8 scale bytes this lane feeds to the MFMAs of the chunk (K-block g of each K-step), packed 4 to a register;
    // those of W sliced (Eq. (6) scale step)
    uint32_t asc[2], wsc[NT][2];
    pack_lane_scales(aslo, ashi, g, asc);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      pack_lane_scales(wslo[nt], wshi[nt], g, wsc[nt]);
      if constexpr (!SLICED) {
        wsc[nt][0] = scale_add_x4(wsc[nt][0], kDeltaE_E4M3_E2M1);
        wsc[nt][1] = scale_add_x4(wsc[nt][1], kDeltaE_E4M3_E2M1);
      }
    }
    if (steps < 8) {   // a K-step that does not exist is multiplied all the same, as zeros under the scale 2^0 (a stray
                       // byte 255 there would turn the exact zero into NaN)
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        if (p >= steps) {
          const uint32_t m = 0xFFu << (8 * (p & 3)), one = 127u << (8 * (p & 3));
          asc[p >> 2] = (asc[p >> 2] & ~m) | one;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) wsc[nt][p >> 2] = (wsc[nt][p >> 2] & ~m) | one;
        }
      }
    }
    wave_lds_order();   // the tile is free again (the reads above execute before the writes below)
    // lane parts of the LDS addresses; the per-row / per-K-step parts are XORed in where they are used (kept opaque so
    // that the compiler does not hold 24 precomputed addresses in registers)
    uint32_t wr_lane = 8u * (uint32_t)lane, rd_lane = 16u * (uint32_t)(g ^ i) + 512u * (uint32_t)i;
    asm volatile("" : "+v"(wr_lane), "+v"(rd_lane));
    static_for<0, NT>([&](auto ntc) {
      constexpr int nt = decltype(ntc)::value;
      // W: lane l holds half l % 2 of block l / 2 of the column's chunk; sliced, it is 8 bytes of the column's row of the
      // tile: slot (l / 2) ^ j, half l % 2
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int r = nt * 16 + j;
        uint32_t half[2];
        if constexpr (SLICED) { half[0] = ring[r % D].x; half[1] = ring[r % D].y; }
        else slice_half_block_e2m1(ring[r % D], half);   // Eq. (6) element step
        *reinterpret_cast<u32x2*>(tile + j * 512 + (wr_lane ^ (16u * j))) = u32x2{half[0], half[1]};
        if (r + D < R) ring[r % D] = load_row(r + D);
        __builtin_amdgcn_sched_barrier(0);
      }
      wave_lds_order();
      // block 4 p + g of column i: slot (4 p + g) ^ i of row i; four K-steps' fragments are read ahead of their MFMAs
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        u32x4 bfr[4];
#pragma unroll
        for (int pp = 0; pp < 4; ++pp) bfr[pp] = *reinterpret_cast<const u32x4*>(tile + (rd_lane ^ (64u * (4 * h + pp))));
#pragma unroll
        for (int pp = 0; pp < 4; ++pp) {
          const i32x8 b = {(int)bfr[pp].x, (int)bfr[pp].y, (int)bfr[pp].z, (int)bfr[pp].w, 0, 0, 0, 0};
          // (the instruction reads the low byte of its scale operands)
          acc[nt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(af[4 * h + pp], b, acc[nt], 0 /* A: E4M3 */, 4 /* B: E2M1 */, 0,
                                                                     (int)(asc[h] >> (8 * pp)), 0, (int)(wsc[nt][h] >> (8 * pp)));
        }
      }
      wave_lds_order();   // the next column tile, or the next chunk's A, overwrites the tile
    });
  }
  if (wave > 0) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) red[((wave - 1) * NT + nt) * 64 + lane] = acc[nt];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const f32x4 r0 = red[(0 * NT + nt) * 64 + lane], r1 = red[(1 * NT + nt) * 64 + lane], r2 = red[(2 * NT + nt) * 64 + lane];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float s = ((acc[nt][j] + r0[j]) + r1[j]) + r2[j];
        const int m = 4 * g + j;
        if (m < M && ncol[nt] < N) c[(int64_t)m * ldc + ncol[nt]] = s;
      }
    }
  }
}

// ------------------------------------------------------------------ 16 < M <= 48: W as in the decode kernel, A as fragments
// The same stream of W (coalesced 1 KB loads, sliced on arrival, a wave-private swizzled LDS tile on the way into the
// operand layout) multiplied with MT row tiles of A.  MT chunks of A do not fit the LDS beside the W tiles, so A comes
// as MFMA operand fragments straight from global memory (it is small and stays in L2; the lanes of such a load sit on 16
// rows, which costs the memory pipe 4 x the time of a coalesced one -- affordable for A, not for W), in groups of
// kGroup K-steps: the first group is requested ahead of W, the second half-way through the slicing, when half of W's
// registers are free, the others (MT > 2) behind the MFMAs of the group whose registers they take.  K is split over
// the four waves in chunks of 1024 as in the decode kernel, and the partial sums are added in the same order.
// SLICED: as in the decode kernel (W is a kept W_t; 8-byte loads, no Slice-and-Scale step, the same bits).
template <int MT, int NT, bool SLICED>
__global__ __launch_bounds__(256, 2) void gemm_fp4_midm_kernel(const uint8_t* __restrict__ a_codes,
                                                               const uint8_t* __restrict__ a_scales,
                                                               const uint8_t* __restrict__ w_codes,
                                                               const uint8_t* __restrict__ w_scales, float* __restrict__ c,
                                                               int M, int N, int K, int64_t ldc) {
  constexpr int kGroups = MT <= 2 ? 2 : 4, kGroup = 8 / kGroups;   // (NT column tiles of 16 per workgroup, as in the decode kernel)
  constexpr int kTile = NT * 8192;   // sliced codes of a chunk: 16 columns x 512 bytes per column tile
  static_assert(3 * MT * NT * 4 * 64 * (int)sizeof(float) <= 4 * kTile, "the partial sums reuse the W tiles");
  extern __shared__ __attribute__((aligned(16))) uint8_t midm_smem[];   // 4 x kTile
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 15, g = lane >> 4;
  const int KB = K / 32, ksteps = K / 128, chunks = (ksteps + 7) / 8;
  uint8_t* tile = midm_smem + wave * kTile;
  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int col0 = blockIdx.x * NT * 16;
  int ncol[NT];   // columns past the edge are computed from column N - 1 and never stored
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) ncol[nt] = col0 + nt * 16 + i;
  // fragment side of A: lane (i, g) <-> row 16 mt + i (rows past M read row M - 1; their products are not stored),
  // bytes 16 g .. and 64 + 16 g .. of each K-step
  const uint8_t* arow[MT];
  uint32_t as_off[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + i < M ? mt * 16 + i : M - 1;
    arow[mt] = a_codes + (int64_t)m * K + 16 * g;
    as_off[mt] = (uint32_t)m * (uint32_t)KB;
  }
  // (the host has checked that W is smaller than 4 GiB; reads past the end of a buffer return zero)
  using WReg = std::conditional_t<SLICED, u32x2, u32x4>;
  constexpr uint32_t kWLane = SLICED ? 8u : 16u, kWChunk = SLICED ? 512u : 1024u;
  const uint32_t w_row = SLICED ? (uint32_t)K / 2u : (uint32_t)K;         // bytes per row of W
  const __amdgpu_buffer_rsrc_t w_rsrc = make_buffer(w_codes, (uint32_t)N * w_row);
  const __amdgpu_buffer_rsrc_t as_rsrc = make_buffer(a_scales, (uint32_t)M * (uint32_t)KB);
  const __amdgpu_buffer_rsrc_t ws_rsrc = make_buffer(w_scales, (uint32_t)N * (uint32_t)KB);
  for (int chunk = wave; chunk < chunks; chunk += 4) {
    const int steps = ksteps - chunk * 8 < 8 ? ksteps - chunk * 8 : 8;
    const uint32_t lane_off = (lane >> 3) < steps ? kWLane * (uint32_t)lane : 0u;   // (as in the decode kernel)
    const uint32_t chunk_off = (uint32_t)chunk * kWChunk;
    // the fragments of A of K-steps kGroup q .. kGroup q + kGroup - 1 of the chunk (a K-step that does not exist: the
    // chunk's last one again, which is not multiplied)
    u32x4 a0[2][kGroup][MT], a1[2][kGroup][MT];
    auto load_a_group = [&](auto qc) __attribute__((always_inline)) {
      constexpr int Q = decltype(qc)::value;
#pragma unroll
      for (int pp = 0; pp < kGroup; ++pp) {
        const int p = Q * kGroup + pp < steps ? Q * kGroup + pp : steps - 1;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const uint8_t* ap = arow[mt] + (int64_t)chunk * 1024 + p * 128;
          a0[Q & 1][pp][mt] = *reinterpret_cast<const u32x4*>(ap);
          a1[Q & 1][pp][mt] = *reinterpret_cast<const u32x4*>(ap + 64);
        }
      }
    };
    // scale bytes (32 per row / column and chunk; in a ragged last chunk they run into the next row or past the end of
    // the array, where a buffer load returns zeros: bytes of K-steps that are not multiplied)
    u32x4 aslo[MT], ashi[MT], wslo[NT], wshi[NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      aslo[mt] = buffer_load_x4<false>(as_rsrc, as_off[mt] + (uint32_t)chunk * 32u, 0u);
      ashi[mt] = buffer_load_x4<false>(as_rsrc, as_off[mt] + (uint32_t)chunk * 32u + 16u, 0u);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const uint32_t wo = (uint32_t)(ncol[nt] < N ? ncol[nt] : N - 1) * (uint32_t)KB + (uint32_t)chunk * 32u;
      wslo[nt] = buffer_load_x4<false>(ws_rsrc, wo, 0u);
      wshi[nt] = buffer_load_x4<false>(ws_rsrc, wo + 16u, 0u);
    }
    load_a_group(std::integral_constant<int, 0>{});
    __builtin_amdgcn_sched_barrier(0);
    WReg wraw[NT][16];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int n = col0 + nt * 16 + j < N ? col0 + nt * 16 + j : N - 1;
        if constexpr (SLICED) wraw[nt][j] = buffer_load_x2<true>(w_rsrc, lane_off, (uint32_t)n * w_row + chunk_off);
        else wraw[nt][j] = buffer_load_x4<true>(w_rsrc, lane_off, (uint32_t)n * w_row + chunk_off);
      }
    __builtin_amdgcn_sched_barrier(0);
    uint32_t asc[MT][2], wsc[NT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) pack_lane_scales(aslo[mt], ashi[mt], g, asc[mt]);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      pack_lane_scales(wslo[nt], wshi[nt], g, wsc[nt]);
      if constexpr (!SLICED) {
        wsc[nt][0] = scale_add_x4(wsc[nt][0], kDeltaE_E4M3_E2M1);   // Eq. (6) scale step
        wsc[nt][1] = scale_add_x4(wsc[nt][1], kDeltaE_E4M3_E2M1);
      }
    }
    // W: lane l holds half l % 2 of block l / 2 of each column's chunk; sliced, it is 8 bytes of the column's row
    static_for<0, NT>([&](auto ntc) {
      constexpr int nt = decltype(ntc)::value;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        uint32_t half[2];
        if constexpr (SLICED) { half[0] = wraw[nt][j].x; half[1] = wraw[nt][j].y; }
        else slice_half_block_e2m1(wraw[nt][j], half);   // Eq. (6) element step
        *reinterpret_cast<u32x2*>(tile + nt * 8192 + j * 512 + 16 * ((lane >> 1) ^ j) + 8 * (lane & 1)) = u32x2{half[0], half[1]};
      }
      if constexpr (nt == 0) {
        __builtin_amdgcn_sched_barrier(0);
        load_a_group(std::integral_constant<int, 1>{});   // half of W's registers are free now
        __builtin_amdgcn_sched_barrier(0);
      }
    });
    wave_lds_order();
    static_for<0, kGroups>([&](auto qc) {
      constexpr int Q = decltype(qc)::value;
#pragma unroll
      for (int pp = 0; pp < kGroup; ++pp) {
        const int p = Q * kGroup + pp;
        if (p < steps) {
          i32x8 b[NT];
          int bscale[NT];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            u32x4 t = *reinterpret_cast<const u32x4*>(tile + nt * 8192 + i * 512 + 16 * ((4 * p + g) ^ i));   // block 4 p + g of column i
            b[nt] = i32x8{(int)t.x, (int)t.y, (int)t.z, (int)t.w, 0, 0, 0, 0};
            bscale[nt] = (int)(wsc[nt][p >> 2] >> (8 * (p & 3)));   // the instruction reads the low byte
          }
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const u32x4 lo = a0[Q & 1][pp][mt], hi = a1[Q & 1][pp][mt];
            const i32x8 a = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
            const int ascale = (int)(asc[mt][p >> 2] >> (8 * (p & 3)));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b[nt], acc[mt][nt], 0 /* A: E4M3 */,
                                                                             4 /* B: E2M1 */, 0, ascale, 0, bscale[nt]);
          }
        }
      }
      // the group after next takes this group's registers
      if constexpr (Q + 2 < kGroups) load_a_group(std::integral_constant<int, Q + 2>{});
    });
    wave_lds_order();   // the next chunk overwrites the tile
  }
  __syncthreads();   // every wave is done with its W tile: the partial sums go where the tiles were
  float(*red)[MT][NT][4][64] = reinterpret_cast<float(*)[MT][NT][4][64]>(midm_smem);   // [3][MT][NT][4][64]
  if (wave > 0) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[wave - 1][mt][nt][j][lane] = acc[mt][nt][j];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float s = ((acc[mt][nt][j] + red[0][mt][nt][j][lane]) + red[1][mt][nt][j][lane]) + red[2][mt][nt][j][lane];
          const int m = mt * 16 + 4 * g + j;
          if (m < M && ncol[nt] < N) c[(int64_t)m * ldc + ncol[nt]] = s;
        }
  }
}

// ------------------------------------------------------------------ large M (prefill): LDS-tiled
// Workgroup tile 256 (M) x 16 NTW (N; NTW = 8, 7 or 6), K-step 128.  Eight waves in two roles, one wave of each role
// per SIMD:
//   waves 0-3, the consumers: each owns 64 rows and all columns of the tile (4 x NTW MFMA tiles); they read
//     fragments from LDS, issue the MFMAs and request the A tile (E4M3, 32 KB per K-step) two K-steps ahead with loads
//     that have LDS as their destination;
//   waves 4-7, the producers: they load the anchor tile of W (up to 16 KB) kGemmWDepth K-steps ahead into registers
//     and slice it to E2M1 (Eq. (6)) on its way into LDS -- once per workgroup instead of once per wave; the tall
//     tile is what amortizes the slicing (about 2.5 vector instructions per element) against the matrix work -- and
//     stage the scale bytes.
// The SIMD's scheduler interleaves the producer's loads and vector work with the consumer's MFMAs; with a
// single role per wave the same work ran back to back (measured: 308 us against 52 us of pure MFMA time).
// LDS holds three K-steps (the one being multiplied, the one being completed, the one being requested), one
// barrier per K-step.  The 16-byte chunks of a row are XOR-swizzled so that the 16 lanes of a lane group hit
// different banks.  The kernel is persistent: one workgroup per compute unit works several tiles in one pipeline.
constexpr int kGemmBM = 256, kGemmBN = 128, kGemmBK = 128;
constexpr int kGemmLdA = 128, kGemmLdB = 64;   // unpadded rows; 16-byte chunks are XOR-swizzled (see GemmStage)
constexpr int kGemmAChunks = kGemmBM * kGemmBK / 16 / 256;   // 16-byte A chunks per producer thread and K-step (8)
constexpr int kGemmThreads = 512;
constexpr int kGemmWDepth = 6;                // K-steps of W in flight per producer thread (weights streaming from HBM:
                                              // 3 -> 182 us, 6 -> 176 us, 10 -> 189 us for 2048 x 14336 x 4096)

// LDS layout of one K-step.  The 16-byte chunk c of row r of A lives at chunk c ^ ((r >> 1) & 7) of that row, chunk c
// of column n of B at chunk c ^ ((n >> 2) & 3): with 64 banks of 4 bytes, the 16 lanes of a 128-bit access then hit 64
// different banks both when a producer writes (8 or 4 consecutive chunks of 2 or 4 consecutive rows) and when a
// consumer reads a fragment (the same chunk of 16 consecutive rows).
struct GemmStage {
  uint8_t a[kGemmBM * kGemmLdA];   // E4M3 codes, row m: 128 bytes of K
  uint8_t b[kGemmBN * kGemmLdB];   // E2M1 codes, column n: 64 bytes (128 nibbles of K)
  uint32_t as[kGemmBM];            // 4 scale bytes per row (one per K-block of the step)
  uint32_t bs[kGemmBN];            // 4 sliced scale bytes per column
};

// s_waitcnt lgkmcnt(0) alone (gfx9 immediate: vmcnt 63 in bits 3:0 and 15:14, expcnt 7 in bits 6:4, lgkmcnt in bits 11:8)
constexpr int kWaitLgkmcnt0 = 15 | (7 << 4) | (0 << 8) | (3 << 14);
constexpr int wait_lgkmcnt0_vmcnt(int v) { return (v & 15) | (7 << 4) | (0 << 8) | ((v >> 4) << 14); }   // s_waitcnt vmcnt(v) lgkmcnt(0)
// A workgroup barrier that is only the instruction; the "memory" clobber keeps the compiler from moving memory
// operations across it.
__device__ __forceinline__ void producer_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Order of the tile list: bands of kGemmBandM M tiles; inside a band the M tile index runs fastest.  A run of
// consecutive list entries is then a block of (up to) 8 M tiles x a few N tiles whatever M is -- with the M tile index
// fastest over ALL of M, a run of 32 entries of a 32-M-tile problem is 32 different A tiles and one W tile, and A
// streams through the L2 once per run (measured at M = 8192: 1.19 against 1.48 PFLOP/s at M = 2048).
constexpr int kGemmBandM = 8;
struct GemmTileShape { int m_tiles, n_tiles, grid; };
__device__ __forceinline__ void gemm_tile_coords(int t, const GemmTileShape& sh, int& tm, int& tn) {
  const int band_tiles = kGemmBandM * sh.n_tiles;
  const int band = t / band_tiles, r = t - band * band_tiles;
  const int left = sh.m_tiles - band * kGemmBandM, h = left < kGemmBandM ? left : kGemmBandM;   // M tiles of this band
  tn = r / h;
  tm = band * kGemmBandM + (r - tn * h);
}
// Position of a role in a workgroup's sequence of K-steps: tile (its place t in the list, its coordinates) and K-step;
// past the last step it stays there (such steps load valid data again that nothing uses).
struct GemmCursor {
  int k, t, tm, tn, tiles_left;
};
__device__ __forceinline__ void gemm_next_tile(GemmCursor& cur, const GemmTileShape& sh) {
  cur.k = 0;
  cur.t += sh.grid;
  gemm_tile_coords(cur.t, sh, cur.tm, cur.tn);
  cur.tiles_left -= 1;
}
__device__ __forceinline__ void gemm_advance(GemmCursor& cur, int ksteps, const GemmTileShape& sh) {
  if (cur.k < ksteps - 1) cur.k += 1;
  else if (cur.tiles_left > 1) gemm_next_tile(cur, sh);
}

// SLICED: W is a W_t the caller keeps (MXFP4 codes, K / 2 bytes per row): the producers load 8 bytes where they would
// have made 8 of 16, and store them as they are; everything else is the same kernel.
template <int NTW, bool SLICED>
__global__ __launch_bounds__(kGemmThreads) void gemm_fp4_tiled_kernel(const uint8_t* __restrict__ a_codes,
                                                                         const uint8_t* __restrict__ a_scales,
                                                                         const uint8_t* __restrict__ w_codes,
                                                                         const uint8_t* __restrict__ w_scales,
                                                                         float* __restrict__ c, int M, int N, int K,
                                                                         int64_t ldc, int m_tiles, int tiles, int k_len,
                                                                         int64_t c_slice) {
  extern __shared__ __attribute__((aligned(16))) uint8_t gemm_smem[];
  GemmStage* stage = reinterpret_cast<GemmStage*>(gemm_smem);
  // K can be split over gridDim.y: slice y multiplies the K elements [y k_len, (y + 1) k_len) of every row -- the
  // last slice what is left of K, at least one K-step -- (K stays the row stride) and writes its partial sums to
  // c + y c_slice.  One slice (k_len = K) is the whole product.
  const uint32_t k_skip = (uint32_t)blockIdx.y * (uint32_t)k_len;
  a_codes += k_skip;
  w_codes += SLICED ? k_skip / 2 : k_skip;
  a_scales += k_skip / 32;
  w_scales += k_skip / 32;
  c += (int64_t)blockIdx.y * c_slice;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // a scalar: the role branch is uniform
  const int tid = threadIdx.x & 255;   // index inside the role's 256 threads
  const int i = lane & 15, g = lane >> 4;
  constexpr int BN = 16 * NTW;   // columns of the workgroup tile
  const int KB = K / 32, ksteps = (K - (int)k_skip < k_len ? K - (int)k_skip : k_len) / kGemmBK;
  // The kernel is persistent: a workgroup works the tiles v, v + gridDim.x, ... of the tile list (bands of 8 M
  // tiles, M tile index fastest inside a band) and both roles run ONE software pipeline over all K-steps of all their tiles: the operands of the next
  // tile's first K-steps are in flight while the current tile is finished, and a consumer goes on to the next tile's
  // MFMAs as soon as it has issued the stores of the finished one.  (A workgroup fills a CU, so with one tile per
  // workgroup nothing overlaps the 4-6 us until a tile's first operands arrive.)
  // Workgroup b runs on XCD b % 8 (round-robin dispatch), and v is chosen so that the workgroups of one XCD take
  // NEIGHBOURING tiles of every round of gridDim.x tiles -- a block of 8 M tiles x a few N tiles -- so that what one of
  // them brings into the XCD's L2 the others use: with v = b an XCD held one M tile and fetched every tile of W.
  const int grid = (int)gridDim.x;
  const int vb = grid % 8 != 0 ? (int)blockIdx.x : ((int)blockIdx.x % 8) * (grid / 8) + (int)blockIdx.x / 8;
  const int my_tiles = (tiles - vb + grid - 1) / grid;   // >= 1: the grid is <= tiles
  const int total = my_tiles * ksteps;                                                     // K-steps of this workgroup
  const GemmTileShape shape = {m_tiles, tiles / m_tiles, grid};
  GemmCursor first = {0, vb, 0, 0, my_tiles};
  gemm_tile_coords(vb, shape, first.tm, first.tn);
  // The two roles run separate loops (so that a wave's registers hold either the accumulators or the prefetched
  // tiles, not both) with the same number of barriers: one after the prologue, one per K-step.
  // Loads return in order within a wave, so the two operands are requested by different waves: W, which comes from HBM
  // or the last-level cache, by the producers, kWDepth K-steps ahead through registers; A, which sits in L2, by the
  // consumers, two K-steps ahead, straight into LDS.  A wave that waits for its A tile then never waits behind a load of
  // W (measured: with both in the producers, the loads of W cost 56 us of the kernel's 194).
  //
  // During K-step k the consumers read stage k % 3 and request A of step k + 2 into stage (k + 2) % 3 -- the stage of
  // step k - 1, which every consumer left at the last barrier; the producers slice W of step k + 1 into stage
  // (k + 1) % 3.  A consumer arrives at the barrier of step k when its reads of stage k have landed and its part of A
  // of step k + 1 is in LDS; a producer when its LDS stores have completed.
  // Tiles of 128 columns leave a consumer no register for the requests of A (it spilled, 20 % slower): there a fifth
  // wave, the loader, requests A and the other three producer waves share W.  The narrower tiles keep the requests in
  // the consumers and four producer waves, which is 2 % faster for them.
  constexpr bool kLoader = NTW == 8;
  if constexpr (kLoader) {
    if (wave == 4) {
      // ---- the A loader: one wave requests the whole A tile (E4M3 codes, 32 KB) and its scale bytes (1 KB) of K-step
      // s + 2 with loads that have LDS as their destination (no registers, no LDS store instructions), waits until
      // those of step s + 1 have landed and arrives at the barrier.  A wave that issues MFMAs never waits for the CU's
      // memory pipe this way (a request held a consumer for ~80 cycles), and the stores of a finished tile share no
      // in-order queue with requests that somebody waits for.
      //   codes: request J (J < 32) is the 1 KB of 16-byte chunks q = lane + 64 J of the tile: row q / 8, position q % 8
      //     in that row of the LDS tile; the hardware puts lane l's 16 bytes at byte 16 l of the block, so the lane
      //     fetches the chunk that the swizzle puts there.
      //   scales: request j (j < 4) is the scale dword of rows 64 j + lane.
      // The buffer descriptors cover the valid rows of ONE tile and the lane offsets are the same for every tile; a row
      // past the edge of A is out of the descriptor's range, which the hardware answers with zeros instead of a read.
      // The whole offset is in the lane register, because the range check looks at that only.  (The host checks
      // 256 K < 2^32.)
      constexpr int kRequests = kGemmBM * kGemmBK / 1024 + kGemmBM / 64;   // 32 + 4 per K-step
      const uint32_t a_lane = (uint32_t)(lane >> 3) * (uint32_t)K + 16u * (uint32_t)((lane & 7) ^ (lane >> 4));
      const uint32_t s_lane = (uint32_t)lane * (uint32_t)KB;
      GemmCursor rq = first;   // the K-step requested next
      auto request_step = [&](int stage_i) __attribute__((always_inline)) {
        const int m0 = rq.tm * kGemmBM;
        const int rows = M - m0 < kGemmBM ? M - m0 : kGemmBM;
        // (the bases are k_skip bytes into row m0, so the descriptors end that much earlier: at the end of the last valid row)
        const __amdgpu_buffer_rsrc_t c_rsrc = make_buffer(a_codes + (int64_t)m0 * K, (uint32_t)rows * (uint32_t)K - k_skip);
        const __amdgpu_buffer_rsrc_t s_rsrc = make_buffer(a_scales + (int64_t)m0 * KB, (uint32_t)rows * (uint32_t)KB - k_skip / 32);
        uint8_t* st = gemm_smem + stage_i * (int)sizeof(GemmStage);
        const uint32_t k_off = (uint32_t)(rq.k * kGemmBK), ks_off = (uint32_t)(rq.k * 4);
        static_for<0, kGemmBM * kGemmBK / 1024>([&](auto jc) {
          constexpr int J = decltype(jc)::value;
          // rows 8 J + lane / 8; their swizzle term (row / 2) % 8 = lane / 16 + 4 (J % 2)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(c_rsrc, (__attribute__((address_space(3))) void*)(st + J * 1024), 16,
                                                   (int)((a_lane ^ (64u * (J & 1))) + (uint32_t)(8 * J) * (uint32_t)K + k_off), 0, 0, 0);
        });
        static_for<0, kGemmBM / 64>([&](auto jc) {
          constexpr int J = decltype(jc)::value;
          __builtin_amdgcn_raw_ptr_buffer_load_lds(s_rsrc, (__attribute__((address_space(3))) void*)(st + offsetof(GemmStage, as) + J * 256), 4,
                                                   (int)(s_lane + (uint32_t)(64 * J) * (uint32_t)KB + ks_off), 0, 0, 0);
        });
        gemm_advance(rq, ksteps, shape);
      };
      // arrive at a barrier when everything but the `kRequests` youngest requests has landed (vector memory operations
      // of a wave complete in the order of issue); no fence, which would wait for those too
      auto arrive = [&] {
        __builtin_amdgcn_s_waitcnt(wait_lgkmcnt0_vmcnt(kRequests));
        producer_barrier();
      };
      request_step(0);
      request_step(1);
      arrive();   // stage 0 is complete
      int st2 = 2;   // (s + 2) % 3: the stage that every consumer left at the last barrier
      for (int s = 0; s < total; ++s) {
        request_step(st2);
        st2 = st2 == 2 ? 0 : st2 + 1;
        arrive();   // step s + 1 is complete
      }
      __builtin_amdgcn_s_waitcnt(0);   // the last requests (of steps that do not exist) must land before the LDS is given back
      return;
    }
  }
  if (wave >= 4) {
    // ---- producers
    //   B: 16-byte piece q = t + PT j (j < WP; PT = 256 producer threads, 192 beside a loader wave) of the anchor tile: column q / 8, half q % 2 of K-block (q % 8) / 2
    //      (16 anchor bytes -> 8 bytes of E2M1), through registers, because it is sliced on the way.  The lanes of a
    //      load read consecutive 16 bytes (8 lanes one 128-byte row).
    //   scales: thread t one row of A (4 bytes; not beside a loader wave); thread t < 16 NTW also one column of W
    // Rows / columns past the edge are clamped to the last valid one instead of branched around: their products
    // land in outputs that are never stored, and straight-line code lets the loads of several K-steps stay in
    // flight (the compiler counts outstanding loads exactly only without control flow).
    constexpr int R = kGemmWDepth;   // register slots: slot s % R holds K-step s from its request until it is staged
    // per-thread parts of the addresses that do not depend on the tile
    constexpr int PT = kLoader ? 192 : 256;        // producer threads
    constexpr int WP = (8 * BN + PT - 1) / PT;     // 16-byte pieces per thread and K-step
    const int pt = kLoader ? (int)threadIdx.x - 320 : tid;
    int w_col[WP], w_piece[WP];
#pragma unroll
    for (int j = 0; j < WP; ++j) {
      const int q = pt + PT * j;
      w_col[j] = (q >> 3) < BN ? (q >> 3) : BN - 1;   // the spare threads of the last piece repeat the tile's last column
      w_piece[j] = (SLICED ? 8 : 16) * (q & 7);
    }
    const int scol = pt < BN ? pt : BN - 1;
    using WReg = std::conditional_t<SLICED, u32x2, u32x4>;   // 16 codes of W as loaded
    const int64_t w_row = SLICED ? K / 2 : K;              // bytes per row of W
    WReg rb[R][WP];
    uint32_t rsa[R], rsw[R];
    GemmCursor ld = first;   // the K-step that the next call of load_step requests
    auto load_step = [&](auto slot_c) __attribute__((always_inline)) {
      constexpr int S = decltype(slot_c)::value;
      const int m0 = ld.tm * kGemmBM, n0 = ld.tn * BN;
      const int k0 = ld.k * (SLICED ? kGemmBK / 2 : kGemmBK);
#pragma unroll
      for (int j = 0; j < WP; ++j) {
        // plain loads: the workgroups that share this W tile run at about the same time, partly on different XCDs,
        // and non-temporal loads made each of them fetch it from HBM (269 us against 196 us for the kernel)
        const int n = n0 + w_col[j] < N ? n0 + w_col[j] : N - 1;
        rb[S][j] = *reinterpret_cast<const WReg*>(w_codes + (int64_t)n * w_row + k0 + w_piece[j]);
      }
      if constexpr (!kLoader) {   // (with a loader wave the scale bytes of A come with its codes)
        const int ms = m0 + pt < M ? m0 + pt : M - 1;
        rsa[S] = *reinterpret_cast<const uint32_t*>(a_scales + (int64_t)ms * KB + ld.k * 4);
      }
      const int ns = n0 + scol < N ? n0 + scol : N - 1;
      rsw[S] = *reinterpret_cast<const uint32_t*>(w_scales + (int64_t)ns * KB + ld.k * 4);
      gemm_advance(ld, ksteps, shape);
    };
    auto store_lds = [&](GemmStage& st, auto slot_c) __attribute__((always_inline)) {
      constexpr int S = decltype(slot_c)::value;
#pragma unroll
      for (int j = 0; j < WP; ++j) {
        const int q = pt + PT * j, col = q >> 3, kb = (q & 7) >> 1, half = q & 1;
        uint32_t b2[2];
        if constexpr (SLICED) { b2[0] = rb[S][j].x; b2[1] = rb[S][j].y; }
        else slice_half_block_e2m1(rb[S][j], b2);   // Eq. (6) element step, once per workgroup and K-step
        // (the spare threads of the last piece, which loaded the tile's last column again, store nothing)
        if (col < BN) *reinterpret_cast<u32x2*>(&st.b[col * kGemmLdB + 16 * (kb ^ ((col >> 2) & 3)) + 8 * half]) = u32x2{b2[0], b2[1]};
      }
      if constexpr (!kLoader) st.as[pt] = rsa[S];
      if (pt < BN) st.bs[pt] = SLICED ? rsw[S] : scale_add_x4(rsw[S], kDeltaE_E4M3_E2M1);   // Eq. (6) scale step
    };
    // prologue: steps 0 .. R - 1 requested, step 0 staged
    static_for<0, R>([&](auto d) { load_step(d); });
    store_lds(stage[0], std::integral_constant<int, 0>{});
    __syncthreads();
    // K-step s: step s + R is requested into the slot that step s left (staged in step s - 1), step s + 1 is staged
    int s1 = 1;   // (s + 1) % 3
    const int rounds = total / R;
    for (int r = 0; r < rounds; ++r) {
      static_for<0, R>([&](auto d) {
        constexpr int DD = decltype(d)::value;
        load_step(d);
        store_lds(stage[s1], std::integral_constant<int, (DD + 1) % R>{});
        s1 = s1 == 2 ? 0 : s1 + 1;
        __syncthreads();
      });
    }
    // the K-steps left over when their number is not a multiple of R (no more loads are needed)
    static_for<0, R - 1>([&](auto d) {
      constexpr int DD = decltype(d)::value;
      if (rounds * R + DD < total) {
        store_lds(stage[s1], std::integral_constant<int, (DD + 1) % R>{});
        s1 = s1 == 2 ? 0 : s1 + 1;
        __syncthreads();
      }
    });
    return;
  }

  // ---- consumers: wave w owns rows m0 + 64 w + [0, 64) and all 16 NTW columns of the tile (4 x NTW MFMA tiles).
  // A K-step goes column tile by column tile, 4 MFMAs each (one per row tile), and every other instruction of the loop
  // sits between two MFMAs -- bunched in front of a group of MFMAs they leave the matrix pipe idle while they issue:
  //   - the B fragments come from LDS through a ring of 4 register sets; the set that a column tile leaves takes the
  //     fragment 4 column tiles further on (of the next K-step, behind the barrier, for the last 4);
  //   - the A fragments of the next K-step (two register sets alternate) are read behind the barrier;
  //   - the requests of A for the step after next go out behind the first MFMAs.
  // The barrier of the step sits where the read-ahead first reaches into the next stage.  Scale bytes are read with
  // byte loads (the instruction takes the low byte of its scale register; a dword load would need a shift that waits
  // for the read).  Scheduling barriers keep the compiler from moving anything back to its use.
  constexpr int MTW = 4, RING = 4;
  static_assert(NTW >= RING && NTW <= kGemmBN / 16, "column tiles per wave");
  f32x4 acc[MTW][NTW];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  // (the tile offsets 64 w, 16 mt, 16 nt do not change the swizzle term of a lane)
  const int a_off = (wave * 64 + i) * kGemmLdA + 16 * (g ^ ((i >> 1) & 7));   // + mt * 16 rows; second run of K: ^ 64
  const int b_off = i * kGemmLdB + 16 * (g ^ ((i >> 2) & 3));                 // + nt * 16 columns
  i32x8 af[2][MTW];   // two 16-byte runs of K per lane
  // B operands: only the low 4 dwords carry FP4 codes; the upper 4 stay zero for the whole kernel
  i32x8 bf[RING];
  uint32_t sa[2][MTW], sb[RING];
#pragma unroll
  for (int r = 0; r < RING; ++r) bf[r] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
  auto read_b = [&](const GemmStage& st, auto nt_c, auto slot_c) {
    constexpr int NT = decltype(nt_c)::value, R = decltype(slot_c)::value;
    u32x4 t = *reinterpret_cast<const u32x4*>(&st.b[b_off + NT * 16 * kGemmLdB]);
    bf[R][0] = (int)t.x; bf[R][1] = (int)t.y; bf[R][2] = (int)t.z; bf[R][3] = (int)t.w;
    sb[R] = reinterpret_cast<const uint8_t*>(st.bs)[(NT * 16 + i) * 4 + g];
  };
  // piece 3 mt + q of a K-step's A fragments: q = 0 / 1 the two 16-byte runs of row tile mt, q = 2 its scale byte
  auto read_a_piece = [&](const GemmStage& st, auto set_c, auto piece_c) {
    constexpr int SET = decltype(set_c)::value, P = decltype(piece_c)::value, mt = P / 3, q = P % 3;
    if constexpr (q == 0) {
      u32x4 t = *reinterpret_cast<const u32x4*>(&st.a[a_off + mt * 16 * kGemmLdA]);
      af[SET][mt][0] = (int)t.x; af[SET][mt][1] = (int)t.y; af[SET][mt][2] = (int)t.z; af[SET][mt][3] = (int)t.w;
    } else if constexpr (q == 1) {
      u32x4 t = *reinterpret_cast<const u32x4*>(&st.a[(a_off ^ 64) + mt * 16 * kGemmLdA]);
      af[SET][mt][4] = (int)t.x; af[SET][mt][5] = (int)t.y; af[SET][mt][6] = (int)t.z; af[SET][mt][7] = (int)t.w;
    } else {
      sa[SET][mt] = reinterpret_cast<const uint8_t*>(st.as)[(wave * 64 + mt * 16 + i) * 4 + g];
    }
  };
  auto mfma_one = [&](auto set_c, auto slot_c, auto mt_c, auto nt_c) {
    constexpr int SET = decltype(set_c)::value, R = decltype(slot_c)::value, MT = decltype(mt_c)::value, NT = decltype(nt_c)::value;
    // W is the instruction's first operand, so a lane's four results are four consecutive COLUMNS of one row of C
    // (one 16-byte store): acc[MT][NT][j] = C[row 16 MT + i][column 16 NT + 4 g + j] of the wave's part of the tile
    acc[MT][NT] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[R], af[SET][MT], acc[MT][NT], 4, 0, 0, (int)sb[R], 0,
                                                                   (int)sa[SET][MT]);
    // (an MFMA has no side effect, so the compiler may move it down into the block of its next use, across the
    // scheduling barriers; the empty statement, which it must not move, holds the result where it is)
    asm volatile("" : "+v"(acc[MT][NT]));
  };
  // A: 16-byte chunk q = tid + 256 j (j < 8) of the tile: row q / 8, position q % 8 in that row of the LDS tile.
  // Requested with LDS as the destination (no registers, no LDS store instruction): the hardware puts lane l's 16
  // bytes at byte 16 l of the wave's 1 KB block, so the lane fetches the chunk that the swizzle puts there.  The
  // buffer descriptor covers the valid rows of ONE tile of A and the lane offsets are the same for every tile; a row
  // past the edge of A is out of the descriptor's range, which the hardware answers with zeros instead of a read.
  // (The host checks 256 K < 2^32.)
  // (Chunk j lies 32 j rows below chunk 0, so one register holds the lane's part and the rest of the offset --
  // 32 j K and the K-step -- is scalar; it is added into the lane offset, not passed as the instruction's scalar
  // offset, because the range check looks at the lane offset only.)
  const uint32_t a_lane = (uint32_t)(tid >> 3) * (uint32_t)K + 16u * (uint32_t)((tid & 7) ^ ((tid >> 4) & 7));
  auto a_tile = [&](const GemmCursor& cur) {
    const int m0 = cur.tm * kGemmBM;
    const int rows = M - m0 < kGemmBM ? M - m0 : kGemmBM;
    return make_buffer(a_codes + (int64_t)m0 * K, (uint32_t)rows * (uint32_t)K - k_skip);   // (ends with the last valid row)
  };
  // K-step ks of the tile behind descriptor rsrc (a step past the end of K: the last one again, which nothing uses)
  auto request_a = [&](__amdgpu_buffer_rsrc_t rsrc, int ks, int stage_i, auto jc) __attribute__((always_inline)) {
    constexpr int J = decltype(jc)::value;
    if constexpr (kLoader) return;   // (the loader wave requests A)
    const int kc = ks < ksteps ? ks : ksteps - 1;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        rsrc, (__attribute__((address_space(3))) void*)(gemm_smem + stage_i * (int)sizeof(GemmStage) + J * 4096 + wave * 1024), 16,
        (int)(a_lane + (uint32_t)(32 * J) * (uint32_t)K + (uint32_t)(kc * kGemmBK)), 0, 0, 0);
  };
  // the barrier of a K-step for a consumer: its LDS reads have landed (the producers overwrite that stage two steps
  // on, the consumers' own requests one step on) and of its requests only the 8 youngest, of the step after next, are
  // still in flight; no fence -- that would wait for those too
  // (`younger`: how many of this wave's requests were issued after those that must have landed -- the ones of the
  // step after next that precede the barrier in the K-step: all 8, or the first 4 with the 64-column tile, whose
  // barrier comes after the fourth MFMA)
  constexpr int kBarrierX = (NTW - RING) * MTW + MTW - 1;   // the MFMA after which the ring first needs the next stage
  constexpr int kYoungerInStep = kBarrierX + 1 < kGemmAChunks ? kBarrierX + 1 : kGemmAChunks;
  auto consumer_barrier = [&](auto younger_c) {
    if constexpr (kLoader) __builtin_amdgcn_s_waitcnt(kWaitLgkmcnt0);   // (the loader waits for A)
    else __builtin_amdgcn_s_waitcnt(wait_lgkmcnt0_vmcnt(decltype(younger_c)::value));
    producer_barrier();
  };
  constexpr int kPieces = 3 * MTW;
  // K-step k with the A fragments in register set SET and B fragment nt in ring slot (PHASE + nt) % RING
  auto k_step = [&](int cur_i, auto set_c, auto phase_c, __amdgpu_buffer_rsrc_t req_rsrc, int req_k) __attribute__((always_inline)) {
    constexpr int SET = decltype(set_c)::value, PHASE = decltype(phase_c)::value;
    using NSET = std::integral_constant<int, SET ^ 1>;
    const int nxt_i = cur_i == 2 ? 0 : cur_i + 1, req_i = cur_i == 0 ? 2 : cur_i - 1;   // (k + 1) % 3, (k + 2) % 3
    const GemmStage& cur = stage[cur_i];
    const GemmStage& nxt = stage[nxt_i];
    static_for<0, NTW * MTW>([&](auto xc) {
      constexpr int X = decltype(xc)::value, NT = X / MTW, MT = X % MTW;
      using SLOT = std::integral_constant<int, (PHASE + NT) % RING>;
      mfma_one(set_c, SLOT{}, std::integral_constant<int, MT>{}, std::integral_constant<int, NT>{});
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (X < kGemmAChunks) {
        request_a(req_rsrc, req_k, req_i, xc);   // A of the step after next, into the stage that every consumer left a step ago
      }
      if constexpr (X == kBarrierX) consumer_barrier(std::integral_constant<int, kYoungerInStep>{});   // every read of this stage has landed; the next one is complete
      if constexpr (MT == MTW - 1) {
        // the ring set of this column tile is free: fragment NT + RING, of this K-step or of the next
        if constexpr (NT + RING < NTW) read_b(cur, std::integral_constant<int, NT + RING>{}, SLOT{});
        else read_b(nxt, std::integral_constant<int, NT + RING - NTW>{}, SLOT{});
      }
      if constexpr (X >= kBarrierX) {
        // behind the barrier: the A fragments of the next K-step, spread over the remaining MFMAs
        constexpr int kLeft = NTW * MTW - kBarrierX;                  // MFMA slots from here on (13)
        constexpr int P0 = (X - kBarrierX) * kPieces / kLeft, P1 = (X - kBarrierX + 1) * kPieces / kLeft;
        static_for<P0, P1>([&](auto pc) { read_a_piece(nxt, NSET{}, pc); });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  // The ring slot of a K-step's first fragment moves on by NTW % RING per step and the A register sets alternate:
  // four K-steps bring both back, so the loop runs in rounds of four with the slots as compile-time constants.
  // Everything that depends on the tile changes BETWEEN rounds: a tile's last K-step is the fourth of a round when K
  // is a multiple of 512, and only then does the host give a workgroup more than one tile.  (Inside a round there
  // must be no control flow at all: the compiler is free to move an MFMA, which has no side effect, down into the
  // block of its next use, and did -- all MFMAs of a round in one clump, their operands spilled.)
  GemmCursor at = first;   // the round being multiplied (k = its first K-step)
  GemmCursor nx = first;   // the round after it
  auto next_round = [&](GemmCursor& cur) {
    if (cur.k + 4 < ksteps) cur.k += 4;
    else if (cur.tiles_left > 1) gemm_next_tile(cur, shape);
    // else: the workgroup's last round; the cursor stays (its requests repeat valid loads that nothing uses)
  };
  next_round(nx);
  __amdgpu_buffer_rsrc_t rs_at = a_tile(at), rs_nx = a_tile(nx);
  static_for<0, kGemmAChunks>([&](auto jc) { request_a(rs_at, 0, 0, jc); });
  static_for<0, kGemmAChunks>([&](auto jc) { request_a(rs_at, 1, 1, jc); });
  consumer_barrier(std::integral_constant<int, kGemmAChunks>{});   // stage 0 is filled (the requests of stage 1 may be in flight)
  static_for<0, kPieces>([&](auto pc) { read_a_piece(stage[0], std::integral_constant<int, 0>{}, pc); });
  static_for<0, RING>([&](auto rc) { read_b(stage[0], rc, rc); });
  __builtin_amdgcn_sched_barrier(0);
  // Stores go through a buffer descriptor that starts at the tile's first element: a lane keeps ONE offset register,
  // (i ldc + 4 g) floats, and the place of each of the 4 NTW row / column tiles is a scalar offset, so the stores
  // need no address registers while the fragments of the next K-step are already held.  (The host checks
  // 256 ldc < 2^30.)
  typedef uint32_t u32v4 __attribute__((ext_vector_type(4)));
  const uint32_t c_lane = ((uint32_t)i * (uint32_t)ldc + (uint32_t)(4 * g)) * 4u;
  auto store_tile = [&]() __attribute__((always_inline)) {
    const int m0 = at.tm * kGemmBM, n0 = at.tn * BN;
    const int rows = M - m0 < kGemmBM ? M - m0 : kGemmBM, cols = N - n0 < BN ? N - n0 : BN;   // the part of the tile inside C
    const __amdgpu_buffer_rsrc_t c_rsrc =
        make_buffer(c + (int64_t)m0 * ldc + n0, ((uint32_t)(rows - 1) * (uint32_t)ldc + (uint32_t)cols) * 4u);
    const int g4 = 4 * g;
    if (rows == kGemmBM && cols == BN) {   // the whole tile lies in C: 16 bytes per lane, no tests
#pragma unroll
      for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
          const f32x4 v = acc[mt][nt];
          __builtin_amdgcn_raw_buffer_store_b128(u32v4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])},
                                                 c_rsrc, (int)c_lane, (int)(((uint32_t)(wave * 64 + mt * 16) * (uint32_t)ldc + (uint32_t)(nt * 16)) * 4u), 0);
        }
    } else {   // a tile on the edge: the 16 x 16 pieces that lie inside C whole as above, the others element by element
               // (lane part against a scalar); pieces wholly outside are skipped
#pragma unroll
      for (int mt = 0; mt < MTW; ++mt) {
        const int rows_left = rows - (wave * 64 + mt * 16);   // rows of C from this piece's first row on (a scalar)
        if (rows_left <= 0) continue;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
          const f32x4 v = acc[mt][nt];
          const int cols_left = cols - nt * 16;
          if (cols_left <= 0) continue;
          const int piece = (int)(((uint32_t)(wave * 64 + mt * 16) * (uint32_t)ldc + (uint32_t)(nt * 16)) * 4u);
          if (rows_left >= 16 && cols_left >= 16) {
            __builtin_amdgcn_raw_buffer_store_b128(u32v4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])},
                                                   c_rsrc, (int)c_lane, piece, 0);
          } else {
            const bool row_ok = i < rows_left;
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (row_ok && g4 < cols_left - j) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[j]), c_rsrc, (int)c_lane, piece + 4 * j, 0);
          }
        }
      }
    }
  };
  constexpr int PH = NTW % RING;
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  int cur_i = 0, s = 0;   // cur_i = s % 3
  auto step_done = [&] { cur_i = cur_i == 2 ? 0 : cur_i + 1; ++s; };
  while (s + 4 <= total) {
    // (requests: two K-steps ahead -- the third and fourth of this round, then the first two of the next)
    k_step(cur_i, C0{}, std::integral_constant<int, 0>{}, rs_at, at.k + 2); step_done();
    k_step(cur_i, C1{}, std::integral_constant<int, PH % RING>{}, rs_at, at.k + 3); step_done();
    k_step(cur_i, C0{}, std::integral_constant<int, (2 * PH) % RING>{}, rs_nx, nx.k); step_done();
    k_step(cur_i, C1{}, std::integral_constant<int, (3 * PH) % RING>{}, rs_nx, nx.k + 1); step_done();
    // a finished tile: stored (the stores drain while the next tile's MFMAs run), and the next one starts from zero.
    // The accumulators are cleared by selects, not inside the branch, so that they stay in place: 128 selects in
    // four K-steps are nothing beside 512 MFMAs.
    const bool done = at.k + 4 == ksteps;
    if (done) store_tile();
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[mt][nt][j] = done ? 0.f : acc[mt][nt][j];
    at = nx; rs_at = rs_nx;
    next_round(nx);
    rs_nx = a_tile(nx);
  }
  if (s < total) {   // the last one to three K-steps of a K that is not a multiple of 512 (the workgroup's only tile)
    k_step(cur_i, C0{}, std::integral_constant<int, 0>{}, rs_at, at.k + 2); step_done();
    if (s < total) { k_step(cur_i, C1{}, std::integral_constant<int, PH % RING>{}, rs_at, at.k + 3); step_done(); }
    if (s < total) { k_step(cur_i, C0{}, std::integral_constant<int, (2 * PH) % RING>{}, rs_at, at.k + 4); step_done(); }
    store_tile();
  }
  __builtin_amdgcn_s_waitcnt(0);   // the last requests (of steps that do not exist) must land before the LDS is given back
}

// ------------------------------------------------------------------ large M, W already sliced: 256 x 256 (or 224) tiles, four waves
// C = DQ(A) * DQ(W_t)^T with W_t = Q_{A->t}(W_A) taken from a workspace (MXFP4 E2M1 codes, K-contiguous, and their
// scale bytes): for large M the conversion is hoisted out of the product -- in the fused kernel above every workgroup
// slices every tile of W it touches, M / 256 times in all, and the slicing waves take half of the CU's registers.
// Without them a workgroup is four waves of 512 registers, one per SIMD: a wave owns 128 x 128 outputs (64 MFMA tiles,
// exactly its 256 accumulation registers), the workgroup 256 x 256, and a K-step brings 50 KB into the CU for 256
// MFMAs where the fused kernel brings 46 KB for 112: the matrix pipe, not the CU's memory pipe, is the longer one.
// Both operands and their scale bytes are requested straight into LDS (no registers, no LDS stores), two K-steps
// ahead, 14 requests per wave and K-step spread between the MFMAs; LDS holds three K-steps; one barrier per K-step
// (no fence: "all but the 14 youngest requests have landed").  A wave goes through its 8 x 8 MFMA tiles row by row:
// the 8 B fragments of a K-step stay in registers, the A fragments pass through two register sets.  The sum over K
// of every output runs in the order of the fused kernel: the results are the same bit for bit.  NTW = 7 makes the
// tile 224 columns wide (a wave owns 128 x 112); the launcher takes it when the grid's rounds then hold fewer MFMAs.
template <int MTW>
struct BigStage {
  uint8_t a[32 * MTW * 128];   // E4M3 codes of the tile's 32 MTW rows, row r: 128 bytes of K, 16-byte chunk c at c ^ ((r >> 1) & 7)
  uint8_t b[256 * 64];         // E2M1 codes, column n: 64 bytes, chunk c at c ^ ((n >> 2) & 3)
  uint32_t as[256];            // 4 scale bytes per row (one per K-block of the step)
  uint32_t bs[256];            // 4 scale bytes per column
};
static_assert(sizeof(BigStage<8>) == 51200 && sizeof(BigStage<4>) == 34816, "stage sizes");
// K-steps held in LDS: three of 50 KB with 256-row tiles; four of 34 KB with 128-row tiles, whose shorter K-steps need
// their operands requested three steps ahead to cover the same latency
template <int MTW>
constexpr int kBigStages = MTW == 8 ? 3 : 4;

// NTW column tiles of 16 per wave: the workgroup tile is 32 NTW columns wide (256 or 224; the launcher takes the width
// whose tiles fill the GPU's rounds better).  MTW row tiles of 16 per wave: the workgroup tile is 32 MTW rows high --
// 256, or 128 for shapes whose 256-row tiles would leave compute units without one (the stage
// is smaller and there is one more of them).
template <int NTW, int MTW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_fp8_fp4_tile256_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales, const uint8_t* __restrict__ w4_codes,
    const uint8_t* __restrict__ w4_scales, float* __restrict__ c, int M, int N, int K, int64_t ldc, int m_tiles, int tiles) {
  extern __shared__ __attribute__((aligned(16))) uint8_t big_smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 15, g = lane >> 4;
  const int wm = wave & 1, wn = wave >> 1;   // the wave's quarter of the tile
  const int KB = K / 32, K2 = K / 2, ksteps = K / 128;
  // tile order as in the fused kernel: bands of 8 M tiles, and the workgroups of one XCD (blockIdx % 8) take neighbours
  const int grid = (int)gridDim.x;
  const int vb = grid % 8 != 0 ? (int)blockIdx.x : ((int)blockIdx.x % 8) * (grid / 8) + (int)blockIdx.x / 8;
  const GemmTileShape shape = {m_tiles, tiles / m_tiles, grid};
  int tm, tn;
  gemm_tile_coords(vb, shape, tm, tn);
  constexpr int BN = 32 * NTW;   // columns of the workgroup tile
  constexpr int BM = 32 * MTW;   // rows of the workgroup tile
  using Stage = BigStage<MTW>;
  constexpr int NS = kBigStages<MTW>;   // stages: K-step s lives in stage s % NS, requested NS - 1 steps ahead
  constexpr int kBigRequests = MTW + 4 + 1 + 1;   // per wave and K-step: MTW KB of A, 4 KB of B, 64 scale dwords of each
  // The requests of a K-step go out behind every other MFMA from the third on (the fifth with 128-row tiles): early in
  // the step, because the barrier of the next step waits for what they bring (from the eleventh MFMA on: 121 against
  // 117-118 us for 2048 x 14336 x 4096; behind every MFMA from the second on: the same).
  constexpr int kRequestX0 = MTW == 8 ? 2 : 4, kRequestStride = 2;
  static_assert(MTW == 8 || MTW == 4, "rows per wave");
  static_assert(kRequestX0 + kRequestStride * (kBigRequests - 1) <= MTW * NTW - 1, "the requests of a K-step fit between its MFMAs");
  const int m0 = tm * BM, n0 = tn * BN;
  const int rows = M - m0 < BM ? M - m0 : BM, cols = N - n0 < BN ? N - n0 : BN;   // the part of the tile inside C
  // descriptors over the valid rows / columns of this tile: what lies past the edge is out of range and reads as zeros
  const __amdgpu_buffer_rsrc_t a_rsrc = make_buffer(a_codes + (int64_t)m0 * K, (uint32_t)rows * (uint32_t)K);
  const __amdgpu_buffer_rsrc_t b_rsrc = make_buffer(w4_codes + (int64_t)n0 * K2, (uint32_t)cols * (uint32_t)K2);
  const __amdgpu_buffer_rsrc_t as_rsrc = make_buffer(a_scales + (int64_t)m0 * KB, (uint32_t)rows * (uint32_t)KB);
  const __amdgpu_buffer_rsrc_t bs_rsrc = make_buffer(w4_scales + (int64_t)n0 * KB, (uint32_t)cols * (uint32_t)KB);
  // lane parts of the offsets (the hardware puts lane l's bytes at 16 l, or 4 l, of the request's LDS block, so the lane
  // fetches the chunk that the swizzle puts there); the whole offset goes into the lane register, which is what the
  // range check looks at
  const uint32_t a_lane = (uint32_t)(lane >> 3) * (uint32_t)K + 16u * (uint32_t)((lane & 7) ^ (lane >> 4));
  const uint32_t b_lane = (uint32_t)(lane >> 2) * (uint32_t)K2 + 16u * (uint32_t)((lane & 3) ^ (lane >> 4));
  const uint32_t s_lane = (uint32_t)(64 * wave + lane) * (uint32_t)KB;
  auto request_one = [&](int kc, uint8_t* st, auto rc) __attribute__((always_inline)) {
    constexpr int R = decltype(rc)::value;
    if constexpr (R < MTW) {
      const int J = wave * MTW + R;   // rows 8 J + lane / 8; their swizzle term (row / 2) % 8 = lane / 16 + 4 (J % 2)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (__attribute__((address_space(3))) void*)(st + J * 1024), 16,
                                               (int)((a_lane ^ (64u * (R & 1))) + (uint32_t)(8 * J) * (uint32_t)K + (uint32_t)(kc * 128)), 0, 0, 0);
    } else if constexpr (R < MTW + 4) {
      const int J = wave * 4 + (R - MTW);   // columns 16 J + lane / 4 (past the tile's width: out of range, zeros); their swizzle term (column / 4) % 4 = lane / 16
      __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (__attribute__((address_space(3))) void*)(st + offsetof(Stage, b) + J * 1024), 16,
                                               (int)(b_lane + (uint32_t)(16 * J) * (uint32_t)K2 + (uint32_t)(kc * 64)), 0, 0, 0);
    } else if constexpr (R == MTW + 4) {   // rows 64 wave + lane (past the tile's height: out of range, zeros)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(as_rsrc, (__attribute__((address_space(3))) void*)(st + offsetof(Stage, as) + wave * 256), 4,
                                               (int)(s_lane + (uint32_t)(kc * 4)), 0, 0, 0);
    } else {                          // columns 64 wave + lane
      __builtin_amdgcn_raw_ptr_buffer_load_lds(bs_rsrc, (__attribute__((address_space(3))) void*)(st + offsetof(Stage, bs) + wave * 256), 4,
                                               (int)(s_lane + (uint32_t)(kc * 4)), 0, 0, 0);
    }
  };
  // (a K-step past the end of K: the last one again, which nothing uses)
  auto request_step = [&](int ks, int stage_i) __attribute__((always_inline)) {
    const int kc = ks < ksteps ? ks : ksteps - 1;
    uint8_t* st = big_smem + stage_i * (int)sizeof(Stage);
    static_for<0, kBigRequests>([&](auto rc) { request_one(kc, st, rc); });
  };
  // my LDS reads have landed (the stage is free) and all requests but those of the youngest NS - 2 K-steps too
  auto arrive = [&] {
    __builtin_amdgcn_s_waitcnt(wait_lgkmcnt0_vmcnt((NS - 2) * kBigRequests));
    producer_barrier();
  };
  f32x4 acc[MTW][NTW];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  // (the tile offsets 16 MTW wm, 16 mt, 16 NTW wn, 16 nt do not change the swizzle term of a lane: 16 NTW / 4 is a multiple of 4)
  static_assert((16 * NTW / 4) % 4 == 0, "swizzle term of the second column half");
  const int a_off = (wm * 16 * MTW + i) * 128 + 16 * (g ^ ((i >> 1) & 7));   // + mt * 16 rows; second run of K: ^ 64
  const int b_off = (wn * 16 * NTW + i) * 64 + 16 * (g ^ ((i >> 2) & 3));    // + nt * 16 columns
  static_for<0, NS - 1>([&](auto sc) { request_step(decltype(sc)::value, decltype(sc)::value); });
  arrive();   // stage 0 is complete
  int cur_i = 0;
  for (int k = 0; k < ksteps; ++k) {
    const int req_i = cur_i == 0 ? NS - 1 : cur_i - 1;   // (k + NS - 1) % NS: the stage that every wave left at the last barrier
    const int kc = k + NS - 1 < ksteps ? k + NS - 1 : ksteps - 1;
    uint8_t* rst = big_smem + req_i * (int)sizeof(Stage);
    const Stage& st = *reinterpret_cast<const Stage*>(big_smem + cur_i * (int)sizeof(Stage));
    i32x8 bf[NTW];   // only the low 4 dwords carry FP4 codes
    uint32_t sb[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) bf[nt] = i32x8{0, 0, 0, 0, 0, 0, 0, 0};
    auto read_b = [&](auto ntc) __attribute__((always_inline)) {
      constexpr int NT = decltype(ntc)::value;
      u32x4 t = *reinterpret_cast<const u32x4*>(&st.b[b_off + NT * 16 * 64]);
      bf[NT][0] = (int)t.x; bf[NT][1] = (int)t.y; bf[NT][2] = (int)t.z; bf[NT][3] = (int)t.w;
      sb[NT] = reinterpret_cast<const uint8_t*>(st.bs)[(wn * 16 * NTW + NT * 16 + i) * 4 + g];
    };
    i32x8 af[2];
    uint32_t sa[2];
    auto read_a = [&](auto mtc) __attribute__((always_inline)) {
      constexpr int MT = decltype(mtc)::value;
      u32x4 t0 = *reinterpret_cast<const u32x4*>(&st.a[a_off + MT * 16 * 128]);
      u32x4 t1 = *reinterpret_cast<const u32x4*>(&st.a[(a_off ^ 64) + MT * 16 * 128]);
      af[MT & 1] = i32x8{(int)t0.x, (int)t0.y, (int)t0.z, (int)t0.w, (int)t1.x, (int)t1.y, (int)t1.z, (int)t1.w};
      sa[MT & 1] = reinterpret_cast<const uint8_t*>(st.as)[(wm * 16 * MTW + MT * 16 + i) * 4 + g];
    };
    read_a(std::integral_constant<int, 0>{});
    read_b(std::integral_constant<int, 0>{});
    read_b(std::integral_constant<int, 1>{});
    read_b(std::integral_constant<int, 2>{});
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, MTW * NTW>([&](auto xc) {
      constexpr int X = decltype(xc)::value, MT = X / NTW, NT = X % NTW;
      // W_t is the instruction's first operand: a lane's four results are four consecutive columns of one row of C
      acc[MT][NT] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[NT], af[MT & 1], acc[MT][NT], 4 /* E2M1 */, 0 /* E4M3 */, 0,
                                                                     (int)sb[NT], 0, (int)sa[MT & 1]);
      asm volatile("" : "+a"(acc[MT][NT]));   // (keeps the result in its accumulation register and the MFMA in its place)
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (MT == 0 && NT + 3 < NTW) read_b(std::integral_constant<int, NT + 3>{});   // B fragments run three MFMAs ahead in the first row
      if constexpr (NT == 1 && MT + 1 < MTW) read_a(std::integral_constant<int, MT + 1>{});   // the next row tile of A, into the other register set
      if constexpr (X >= kRequestX0 && X < kRequestX0 + kRequestStride * kBigRequests && (X - kRequestX0) % kRequestStride == 0)
        request_one(kc, rst, std::integral_constant<int, (X - kRequestX0) / kRequestStride>{});
      __builtin_amdgcn_sched_barrier(0);
    });
    arrive();   // K-step k + 1 is complete
    cur_i = cur_i == NS - 1 ? 0 : cur_i + 1;
  }
  __builtin_amdgcn_s_waitcnt(0);   // the last requests (of steps that do not exist) must land before the LDS is given back
  // acc[mt][nt][j] = C[row 16 mt + i][column 16 nt + 4 g + j] of the wave's quarter
  float* ct = c + (int64_t)(m0 + wm * 16 * MTW + i) * ldc + n0 + wn * 16 * NTW + 4 * g;
  if (rows == BM && cols == BN) {
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) *reinterpret_cast<f32x4*>(ct + (int64_t)(mt * 16) * ldc + nt * 16) = acc[mt][nt];
  } else {   // a tile on the edge: the 16 x 16 pieces that lie inside C whole as above, the ragged ones element by element
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
      const int rows_left = rows - (wm * 16 * MTW + mt * 16);   // (scalars: the branches are uniform)
      if (rows_left <= 0) continue;
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        const int cols_left = cols - (wn * 16 * NTW + nt * 16);
        if (cols_left <= 0) continue;
        float* piece = ct + (int64_t)(mt * 16) * ldc + nt * 16;
        f32x4 v = acc[mt][nt];
        asm volatile("" : "+v"(v));   // (one piece leaves its accumulation registers at a time; all 64 at once spill)
        if (rows_left >= 16 && cols_left >= 16) {
          *reinterpret_cast<f32x4*>(piece) = v;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (i < rows_left && 4 * g + j < cols_left) piece[j] = v[j];
        }
      }
    }
  }
}

// Two facts about a device are memoized, per device and safely under concurrent callers (atomics; both are
// properties that never change, and asking or setting twice is harmless): its number of compute units, and that a
// kernel has been allowed its dynamic LDS size there (hipFuncSetAttribute acts on the current device).
static int current_device() {
  int dev = 0;
  return hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64 ? dev : -1;
}
static int device_compute_units() {   // 0 on failure
  static std::atomic<int> cu_count[64];
  const int dev = current_device();
  if (dev < 0) return 0;
  int n = cu_count[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
    cu_count[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}
template <auto Kernel>
static bool allow_dynamic_lds(int bytes) {
  static std::atomic<uint64_t> done{0};   // bit d: set on device d
  const int dev = current_device();
  if (dev < 0) return false;
  if (done.load(std::memory_order_acquire) >> dev & 1u) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return false;
  done.fetch_or((uint64_t)1 << dev, std::memory_order_release);
  return true;
}

// The streaming kernels (M <= 48; they address W, and the decode kernel its up to 16 rows of A, with 32-bit offsets).
// Returns false, with nothing enqueued, when the shape is not theirs.  SLICED: W holds MXFP4 codes, K / 2 bytes per row.
template <bool SLICED>
static bool gemm_stream_launch(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                               float* c, int64_t M, int64_t N, int64_t K, int64_t ldc, hipStream_t stream, mx_status_t* status) {
  const bool w_fits_32_bits = N * (SLICED ? K / 2 : K) <= 0xFFFFFFFFll && 16 * K <= 0xFFFFFFFFll;
  if (M > kMidmMaxM || !w_fits_32_bits) return false;
  *status = MX_ERR_LAUNCH;
  const int cus = device_compute_units();
  if (cus <= 0) return true;
  if (M > 16) {
    const int mt_mid = (int)((M + 15) / 16), nt_mid = (N + 31) / 32 >= cus ? 2 : 1;   // (16 columns per workgroup when 32 leave compute units idle)
#define MX_GEMM_MIDM(MT, NT)                                                                                               \
  if (mt_mid == MT && nt_mid == NT) {                                                                                      \
    constexpr int kSmem = 4 * NT * 8192;                                                                                   \
    if (!allow_dynamic_lds<gemm_fp4_midm_kernel<MT, NT, SLICED>>(kSmem)) return true;                                       \
    hipLaunchKernelGGL((gemm_fp4_midm_kernel<MT, NT, SLICED>), dim3((unsigned)((N + 16 * NT - 1) / (16 * NT))), dim3(256), \
                       kSmem, stream, a_codes, a_scales, w_codes, w_scales, c, (int)M, (int)N, (int)K, ldc);              \
  }
    MX_GEMM_MIDM(2, 2) MX_GEMM_MIDM(3, 2) MX_GEMM_MIDM(2, 1) MX_GEMM_MIDM(3, 1)
#undef MX_GEMM_MIDM
  } else {
    // 32 columns per workgroup; 16 when 32 would leave compute units without one (N = 4096, K = 14336: 27 us with 128
    // workgroups of 32 columns)
#define MX_GEMM_DECODE(NT)                                                                                                  \
  {                                                                                                                         \
    if (!allow_dynamic_lds<gemm_fp4_decode_kernel<NT, SLICED>>(decode_smem_bytes(NT))) return true;                         \
    hipLaunchKernelGGL((gemm_fp4_decode_kernel<NT, SLICED>), dim3((unsigned)((N + 16 * NT - 1) / (16 * NT))), dim3(256),    \
                       decode_smem_bytes(NT), stream, a_codes, a_scales, w_codes, w_scales, c, (int)M, (int)N, (int)K, ldc); \
  }
    if ((N + 31) / 32 >= cus) MX_GEMM_DECODE(2) else MX_GEMM_DECODE(1)
#undef MX_GEMM_DECODE
  }
  *status = launch_status(SLICED ? "the MXFP8 x MXFP4 GEMM" : "the fused GEMM");
  return true;
}

// The tiled kernel: any M (below 49 rows only when W has 4 GiB or more).
template <bool SLICED>
static mx_status_t gemm_tiled_launch(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                                     const uint8_t* w_scales, float* c, int64_t M, int64_t N, int64_t K, int64_t ldc,
                                     hipStream_t stream) {
  if (kGemmBM * K > 0xFFFFFFFFll) return MX_ERR_UNSUPPORTED;   // the kernel addresses a tile of A with 32-bit offsets
  const int cus = device_compute_units();
  if (cus <= 0) return MX_ERR_LAUNCH;
  // Tile width: one workgroup fills a CU, so the tiles run in rounds of `cus`; the narrower tiles trade work per
  // tile for a last round that is less empty, or for more workgroups when M is small.  A tile costs a fixed part (its
  // A tile and the latencies of a K-step do not shrink with the width) plus a part per column: measured 19 us + 0.26 us
  // per column for K = 4096, hence cost ~ rounds x (5 + width / 16).  (896 tiles of 128 columns on 256 CUs are 4
  // rounds of which the last is half empty; 1024 tiles of 112 columns are 4 full rounds of 7/8 the work.  M = 128:
  // 224 tiles of 64 columns take 36 us, 128 tiles of 112 columns 48 us.)
  const int64_t m_tiles = (M + kGemmBM - 1) / kGemmBM;
  int ntw = 8;
  int64_t best = -1;
  for (int cand = 8; cand >= 4; --cand) {
    const int64_t tiles_c = m_tiles * ((N + 16 * cand - 1) / (16 * cand));
    const int64_t cost = (tiles_c + cus - 1) / cus * (50 + cand * 10);
    if (best < 0 || cost < best) { best = cost; ntw = cand; }
  }
  const int64_t n_tiles = (N + 16 * ntw - 1) / (16 * ntw);
  const int64_t tiles = m_tiles * n_tiles;
  if (tiles > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  // one persistent workgroup per CU (its LDS and registers fill the CU), fewer when there are fewer tiles; the kernel
  // counts the K-steps of a workgroup in an int
  const int64_t grid_wgs = (tiles < cus || K % (4 * kGemmBK) != 0) ? tiles : cus;   // (the kernel takes several tiles only in rounds of four K-steps)
  if ((tiles + grid_wgs - 1) / grid_wgs * (K / kGemmBK) > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
  if (ldc * kGemmBM >= ((int64_t)1 << 30)) return MX_ERR_UNSUPPORTED;   // a tile of C is addressed with 32-bit byte offsets
  // 3 stages x 41.5 KB: above the 64 KB a kernel gets by default, so the dynamic size is requested explicitly
  constexpr int kSmem = 3 * (int)sizeof(GemmStage);
#define MX_GEMM_TILED(NTW)                                                                                                  \
  if (ntw == NTW) {                                                                                                         \
    if (!allow_dynamic_lds<gemm_fp4_tiled_kernel<NTW, SLICED>>(kSmem)) return MX_ERR_LAUNCH;                                \
    hipLaunchKernelGGL((gemm_fp4_tiled_kernel<NTW, SLICED>), dim3((unsigned)grid_wgs), dim3(kGemmThreads), kSmem, stream, \
                       a_codes, a_scales, w_codes, w_scales, c, (int)M, (int)N, (int)K, ldc, (int)m_tiles, (int)tiles,      \
                       (int)K, (int64_t)0);                                                                                \
  }
  MX_GEMM_TILED(8) MX_GEMM_TILED(7) MX_GEMM_TILED(6) MX_GEMM_TILED(5) MX_GEMM_TILED(4)
#undef MX_GEMM_TILED
  return launch_status(SLICED ? "the MXFP8 x MXFP4 GEMM" : "the fused GEMM");
}

mx_status_t gemm_ss_fp4_launch(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                               const uint8_t* w_scales, float* c, int64_t M, int64_t N, int64_t K, int64_t ldc,
                               hipStream_t stream) {
  mx_status_t status;
  if (gemm_stream_launch<false>(a_codes, a_scales, w_codes, w_scales, c, M, N, K, ldc, stream, &status)) return status;
  return gemm_tiled_launch<false>(a_codes, a_scales, w_codes, w_scales, c, M, N, K, ldc, stream);
}

// C = the K slices' partial sums added in the order of the slices: thread q takes 4 consecutive columns of one row.
// (The partial sums lie in S slices of M x ldp floats, ldp = N rounded up to 4; the padding columns are never written
// by the product and never stored here.)
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const float* __restrict__ p, float* __restrict__ c, int M,
                                                                 int N, int ldp, int64_t ldc, int64_t slice, int S) {
  const int quads = ldp / 4;
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= (int64_t)M * quads) return;
  const int m = (int)(q / quads), n = (int)(q - (int64_t)m * quads) * 4;
  const float* src = p + (int64_t)m * ldp + n;
  f32x4 sum = *reinterpret_cast<const f32x4*>(src);
  for (int s = 1; s < S; ++s) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(src + (int64_t)s * slice);
    sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
  }
  float* dst = c + (int64_t)m * ldc + n;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (n + j < N) dst[j] = sum[j];
}

// The tiled kernel with K split over several workgroups per tile, for shapes whose tiles leave most compute units
// without one (49 <= M and a narrow N: 64 x 4096 x 14336 is 64 tiles of 112 K-steps each on 256 CUs).  Slice s of a
// tile sums its K / S elements in the usual order into a buffer of partial sums in the workspace; a second kernel
// adds the S partial sums of every output in the order of the slices -- a fixed order, but not the one of the
// unsplit kernels.  gemm_splitk_slices is the plan (1: no split, because it does not pay or does not fit);
// gemm_ss_fp4_splitk returns false, with nothing enqueued, when the plan is 1.
int gemm_splitk_slices(int64_t M, int64_t N, int64_t K, size_t workspace_bytes, int* ntw_out) {
  if (M <= kMidmMaxM) return 1;   // (the streaming kernels split K inside a workgroup)
  if (kGemmBM * K > 0xFFFFFFFFll) return 1;
  const int cus = device_compute_units();
  if (cus <= 0) return 1;
  const int64_t ksteps = K / kGemmBK, m_tiles = (M + kGemmBM - 1) / kGemmBM, ldp = (N + 3) & ~(int64_t)3;
  if (ldp * kGemmBM >= ((int64_t)1 << 30)) return 1;
  // The split pays when the narrowest tiles still leave half of the compute units without one: with more workgroups
  // than that the unsplit launch is already bound by the stream of W (64 x 14336 x 4096, 224 tiles of 64 columns: 25.7
  // us unsplit, 28.8 us in two slices), with fewer it is bound by the K-steps one workgroup makes in sequence
  // (64 x 4096 x 14336, 64 tiles: 71 us unsplit, 33 us in eight slices).
  if (m_tiles * ((N + 63) / 64) > cus / 2) return 1;
  // cost of a launch in units of ~12 ns: a K-step of a tile of 16 w columns takes (50 + 10 w) (the model of the
  // unsplit launch), a workgroup's launch, way to its first operands and last stores ~750 (9 us measured), the second
  // kernel and the gap in front of it ~420 (5 us)
  int best_s = 1, best_ntw = 0;
  int64_t best = -1;
  for (int cand = 8; cand >= 4; --cand) {
    const int64_t tiles_c = m_tiles * ((N + 16 * cand - 1) / (16 * cand));
    const int64_t cost = (tiles_c + cus - 1) / cus * ksteps * (50 + cand * 10) + 750;
    if (best < 0 || cost < best) { best = cost; best_ntw = cand; }
  }
  for (int S = 2; S <= 8; ++S) {
    const int64_t per = (ksteps + S - 1) / S;                                            // K-steps of a slice; the last one takes the rest
    if (per < 8 || (S - 1) * per >= ksteps) continue;                                    // slices of eight K-steps and more, none empty
    if ((uint64_t)S * (uint64_t)M * (uint64_t)ldp * 4u > (uint64_t)workspace_bytes) continue;
    for (int cand = 8; cand >= 4; --cand) {
      const int64_t tiles_c = m_tiles * ((N + 16 * cand - 1) / (16 * cand));
      if (tiles_c * S > cus) continue;                                                   // one round
      const int64_t cost = per * (20 + cand * 15) + 750 + 420;   // (with every CU at work a wide tile's K-step costs more: 256 x 4096 x 14336 in 7 slices of 128 columns 42 us, in 4 of 64 columns 39 us)
      if (cost < best) { best = cost; best_s = S; best_ntw = cand; }
    }
  }
  if (ntw_out) *ntw_out = best_ntw;
  return best_s;
}

template <bool SLICED>
static bool gemm_splitk_launch(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                               float* c, int64_t M, int64_t N, int64_t K, int64_t ldc, void* workspace, size_t workspace_bytes,
                               hipStream_t stream, mx_status_t* status) {
  int ntw = 0;
  const int S = gemm_splitk_slices(M, N, K, workspace_bytes, &ntw);
  if (S == 1) return false;
  const int64_t m_tiles = (M + kGemmBM - 1) / kGemmBM, ldp = (N + 3) & ~(int64_t)3;
  const int64_t tiles = m_tiles * ((N + 16 * ntw - 1) / (16 * ntw));
  const int64_t k_len = (K / kGemmBK + S - 1) / S * kGemmBK, slice = M * ldp;
  float* partial = static_cast<float*>(workspace);
  constexpr int kSmem = 3 * (int)sizeof(GemmStage);
  *status = MX_ERR_LAUNCH;
#define MX_GEMM_TILED_SPLIT(NTW)                                                                                            \
  if (ntw == NTW) {                                                                                                         \
    if (!allow_dynamic_lds<gemm_fp4_tiled_kernel<NTW, SLICED>>(kSmem)) return true;                                         \
    hipLaunchKernelGGL((gemm_fp4_tiled_kernel<NTW, SLICED>), dim3((unsigned)tiles, (unsigned)S), dim3(kGemmThreads), kSmem, \
                       stream, a_codes, a_scales, w_codes, w_scales, partial, (int)M, (int)N, (int)K, ldp, (int)m_tiles,    \
                       (int)tiles, (int)k_len, slice);                                                                      \
  }
  MX_GEMM_TILED_SPLIT(8) MX_GEMM_TILED_SPLIT(7) MX_GEMM_TILED_SPLIT(6) MX_GEMM_TILED_SPLIT(5) MX_GEMM_TILED_SPLIT(4)
#undef MX_GEMM_TILED_SPLIT
  if ((*status = launch_status("the fused GEMM (K slices)")) != MX_OK) return true;
  const int64_t quads = M * (ldp / 4);
  hipLaunchKernelGGL(gemm_splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, partial, c, (int)M,
                     (int)N, (int)ldp, ldc, slice, S);
  *status = launch_status("the sum of the fused GEMM's K slices");
  return true;
}

bool gemm_ss_fp4_splitk(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                        float* c, int64_t M, int64_t N, int64_t K, int64_t ldc, void* workspace, size_t workspace_bytes,
                        hipStream_t stream, mx_status_t* status) {
  return gemm_splitk_launch<false>(a_codes, a_scales, w_codes, w_scales, c, M, N, K, ldc, workspace, workspace_bytes, stream, status);
}
bool gemm_fp8_fp4_splitk(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w4_codes, const uint8_t* w4_scales,
                         float* c, int64_t M, int64_t N, int64_t K, int64_t ldc, void* workspace, size_t workspace_bytes,
                         hipStream_t stream, mx_status_t* status) {
  return gemm_splitk_launch<true>(a_codes, a_scales, w4_codes, w4_scales, c, M, N, K, ldc, workspace, workspace_bytes, stream, status);
}

// Do tiles of 256 rows (256 columns wide) give at least 3/4 of the compute units a workgroup?
static bool gemm_tall_tiles_fill(int64_t M, int64_t N, int cus) {
  return 4 * (((M + 255) / 256) * ((N + 255) / 256)) >= 3 * (int64_t)cus;
}

// Is the product with W sliced beforehand the faster one?  Its tiles must fill the GPU: measured on 256 CUs, 192 tiles
// of 256 x 256 win (2048 x 6144 x 4096: 60 against 68 us), 128 and 112 such tiles lose (2048 x 4096 x 4096: 56 against
// 48 us; 512 x 14336 x 4096: 67 against 46 us).  There tiles of 128 rows fill the GPU, with less work per byte of
// operand; they win from 1024 rows on (2048 x 4096 x 4096: 46 against 48 us, 2048 x 4096 x 14336: 134 against 146 us)
// and lose below, where the conversion pass is a larger part of the call (512 x 14336 x 4096: 55 against 46 us).
bool gemm_hoist_pays(int64_t M, int64_t N) {
  const int cus = device_compute_units();
  if (cus <= 0) return false;
  return gemm_tall_tiles_fill(M, N, cus) || (M >= 1024 && 4 * (((M + 127) / 128) * ((N + 255) / 256)) >= 3 * (int64_t)cus);
}

// With W already MXFP4 in memory there is no conversion pass to weigh against: the four-wave kernel with tiles of 256
// (or 128) rows x 256 columns takes the product as soon as such tiles give 3/4 of the compute units a workgroup;
// below that the eight-wave kernel with its narrower tiles (and several tiles per workgroup) does.
bool gemm_big_tiles_pay(int64_t M, int64_t N) {
  const int cus = device_compute_units();
  if (cus <= 0) return false;
  return gemm_tall_tiles_fill(M, N, cus) || 4 * (((M + 127) / 128) * ((N + 255) / 256)) >= 3 * (int64_t)cus;
}

// The product with W already sliced (E2M1 codes [N][K / 2] and scale bytes [N][K / 32], a workspace's or the caller's).
mx_status_t gemm_fp8_fp4_launch(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w4_codes,
                                const uint8_t* w4_scales, float* c, int64_t M, int64_t N, int64_t K, int64_t ldc,
                                hipStream_t stream) {
  mx_status_t status;
  if (gemm_stream_launch<true>(a_codes, a_scales, w4_codes, w4_scales, c, M, N, K, ldc, stream, &status)) return status;
  if (!gemm_big_tiles_pay(M, N)) return gemm_tiled_launch<true>(a_codes, a_scales, w4_codes, w4_scales, c, M, N, K, ldc, stream);
  if (256 * K > 0xFFFFFFFFll) return MX_ERR_UNSUPPORTED;   // a tile is addressed with 32-bit offsets
  const int cus = device_compute_units();
  if (cus <= 0) return MX_ERR_LAUNCH;
  // tile height 256, or 128 when tiles of 256 rows would leave a quarter of the compute units or more without one
  // (2048 x 4096: 128 tiles of 256 x 256, 256 of 128 x 256); tile width 256 or 224: rounds on the GPU x width
  // (2048 x 14336: 448 tiles of 256 columns are 1.75 rounds that take 2, 512 tiles of 224 columns two full rounds of
  // 7/8 the work)
  const bool low = !gemm_tall_tiles_fill(M, N, cus);
  const int64_t m_tiles = low ? (M + 127) / 128 : (M + 255) / 256;
  const int64_t t8 = m_tiles * ((N + 255) / 256), t7 = m_tiles * ((N + 223) / 224);
  const bool narrow = (t7 + cus - 1) / cus * 7 < (t8 + cus - 1) / cus * 8;
  const int64_t tiles = narrow ? t7 : t8;
  if (tiles > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
#define MX_GEMM_TILE256(NTW, MTW)                                                                                           \
  {                                                                                                                         \
    constexpr int kSmem = kBigStages<MTW> * (int)sizeof(BigStage<MTW>);                                                     \
    if (!allow_dynamic_lds<gemm_fp8_fp4_tile256_kernel<NTW, MTW>>(kSmem)) return MX_ERR_LAUNCH;                             \
    hipLaunchKernelGGL((gemm_fp8_fp4_tile256_kernel<NTW, MTW>), dim3((unsigned)tiles), dim3(256), kSmem, stream, a_codes,   \
                       a_scales, w4_codes, w4_scales, c, (int)M, (int)N, (int)K, ldc, (int)m_tiles, (int)tiles);            \
  }
  if (low) {
    if (narrow) MX_GEMM_TILE256(7, 4) else MX_GEMM_TILE256(8, 4)
  } else {
    if (narrow) MX_GEMM_TILE256(7, 8) else MX_GEMM_TILE256(8, 8)
  }
#undef MX_GEMM_TILE256
  return launch_status("the MXFP8 x MXFP4 GEMM");
}

}  // namespace mx
