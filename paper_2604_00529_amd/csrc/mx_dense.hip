// Dense <-> packed kernels: MX quantization (Eq. (1), (2)), dequantization (V^ = X * P) and the
// fused quantize-dequantize of the QAT forward pass (Sec. 3.2; Eq. (7) when an anchor is given).
//
// Blocks along a row (axis 1): one lane owns one 16-byte chunk of the dense tensor (4 fp32 or
// 8 bf16), a block is 8 or 4 adjacent lanes.  The block maximum is reduced with DPP lane
// permutes (no LDS), every lane converts its own elements, and sub-dword code pieces are merged
// across neighbouring lanes with DPP so that the stores are whole dwords.
// Blocks down a column (axis 0): one lane owns 4 adjacent columns over the 32 rows of a block
// (32 coalesced row loads held in registers); no cross-lane step at all.
#include "mx_device.h"
#include "mx_launch.h"

namespace mx {

// Streaming accesses: every input is read once and every output written once per launch.  Non-temporal
// loads and stores are worth two to five points of HBM bandwidth here, and far more with several chunks per lane.
template <typename T>
__device__ __forceinline__ T stream_load(const T* p) {
  return __builtin_nontemporal_load(p);
}
template <typename T>
__device__ __forceinline__ void stream_store(T* p, T v) {
  __builtin_nontemporal_store(v, p);
}

// ------------------------------------------------------------------ dense chunks
template <int DT> struct Dense;
template <> struct Dense<MX_F32> { static constexpr int N = 4, ESZ = 4; };
template <> struct Dense<MX_BF16> { static constexpr int N = 8, ESZ = 2; };

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 p = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, p);
}

// 16-byte chunk at element offset `off` -> N floats
template <int DT>
__device__ __forceinline__ void load_chunk(const void* base, int64_t off, float (&v)[Dense<DT>::N]) {
  u32x4 t = stream_load(reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + off * Dense<DT>::ESZ));
  if constexpr (DT == MX_F32) {
    v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y); v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
  } else {
    v[0] = bf16_lo(t.x); v[1] = bf16_hi(t.x); v[2] = bf16_lo(t.y); v[3] = bf16_hi(t.y);
    v[4] = bf16_lo(t.z); v[5] = bf16_hi(t.z); v[6] = bf16_lo(t.w); v[7] = bf16_hi(t.w);
  }
}

template <int DT>
__device__ __forceinline__ void store_chunk(void* base, int64_t off, const float (&v)[Dense<DT>::N]) {
  u32x4 t;
  if constexpr (DT == MX_F32) {
    t = u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
  } else {
    t = u32x4{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
  }
  stream_store(reinterpret_cast<u32x4*>(static_cast<char*>(base) + off * Dense<DT>::ESZ), t);
}

// 4 elements (one lane's columns of one row) for the column-axis kernels: 16 B fp32 / 8 B bf16
template <int DT>
__device__ __forceinline__ void load_quad(const void* base, int64_t off, float (&v)[4]) {
  if constexpr (DT == MX_F32) {
    u32x4 t = stream_load(reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + off * 4));
    v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y); v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
  } else {
    u32x2 t = stream_load(reinterpret_cast<const u32x2*>(static_cast<const char*>(base) + off * 2));
    v[0] = bf16_lo(t.x); v[1] = bf16_hi(t.x); v[2] = bf16_lo(t.y); v[3] = bf16_hi(t.y);
  }
}

template <int DT>
__device__ __forceinline__ void store_quad(void* base, int64_t off, const float (&v)[4]) {
  if constexpr (DT == MX_F32) {
    stream_store(reinterpret_cast<u32x4*>(static_cast<char*>(base) + off * 4),
                 u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])});
  } else {
    stream_store(reinterpret_cast<u32x2*>(static_cast<char*>(base) + off * 2), u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])});
  }
}

// ------------------------------------------------------------------ cross-lane helpers (DPP, no LDS)
template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
constexpr int DPP_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i <-> 7 - i inside each group of 8
constexpr int DPP_ROW_SHL1 = 0x101;    // lane i reads lane i + 1 (inside a row of 16)

// maximum over the G (4 or 8) adjacent lanes that share a block; every lane gets the result
template <int G>
__device__ __forceinline__ uint32_t group_max(uint32_t m) {
  uint32_t o = dpp<DPP_XOR1>(m); m = m > o ? m : o;
  o = dpp<DPP_XOR2>(m); m = m > o ? m : o;
  if constexpr (G == 8) { o = dpp<DPP_HALF_MIRROR>(m); m = m > o ? m : o; }
  return m;
}

// the same for a block size chosen at run time: `lanes` = 2, 4, 8, 16 or 32 adjacent lanes per block (wave-uniform)
constexpr int DPP_ROW_MIRROR = 0x140;  // lane i <-> 15 - i inside each row of 16
__device__ __forceinline__ uint32_t group_max_lanes(uint32_t m, int lanes) {
  uint32_t o = dpp<DPP_XOR1>(m); m = m > o ? m : o;
  if (lanes >= 4) { o = dpp<DPP_XOR2>(m); m = m > o ? m : o; }
  if (lanes >= 8) { o = dpp<DPP_HALF_MIRROR>(m); m = m > o ? m : o; }
  if (lanes >= 16) { o = dpp<DPP_ROW_MIRROR>(m); m = m > o ? m : o; }
  if (lanes >= 32) { o = (uint32_t)__shfl_xor((int)m, 16, 64); m = m > o ? m : o; }
  return m;
}
// KG = false: blocks of 32 (group size known at compile time); KG = true: 2^log2_lanes lanes per block
template <int G, bool KG>
__device__ __forceinline__ uint32_t block_max(uint32_t m, int log2_lanes) {
  if constexpr (KG) return group_max_lanes(m, 1 << log2_lanes);
  else return group_max<G>(m);
}

template <int N>
__device__ __forceinline__ uint32_t chunk_amax_bits(const float (&v)[N]) {
  uint32_t m = 0;
#pragma unroll
  for (int i = 0; i < N; ++i) { uint32_t a = abs_bits(v[i]); m = m > a ? m : a; }
  return m;
}

// ------------------------------------------------------------------ chunk index -> element offset
// Chunk q of a [rows, cols] matrix (cols / N chunks per row).  flat: ld == cols.
template <int N>
__device__ __forceinline__ int64_t chunk_offset(int64_t q, uint32_t chunks_per_row, int64_t ld, bool flat) {
  if (flat) return q * N;
  uint32_t row = (uint32_t)((uint64_t)q / chunks_per_row);
  uint32_t c = (uint32_t)((uint64_t)q - (uint64_t)row * chunks_per_row);
  return (int64_t)row * ld + (int64_t)c * N;
}

// ------------------------------------------------------------------ axis 1: quantize
// Store the N * W code bits of this lane's chunk.  `lig` = lane index inside the block's group.
template <int W, int N>
__device__ __forceinline__ void store_chunk_codes(uint32_t* block_words, uint64_t bits, int lig) {
  constexpr int NB = N * W;  // bits per lane
  if constexpr (NB == 64) {
    stream_store(reinterpret_cast<u32x2*>(block_words + 2 * lig), u32x2{(uint32_t)bits, (uint32_t)(bits >> 32)});
  } else if constexpr (NB == 32) {
    stream_store(block_words + lig, (uint32_t)bits);
  } else if constexpr (NB == 16) {
    // pairs of lanes make one dword; the even lane stores
    uint32_t nxt = dpp<DPP_ROW_SHL1>((uint32_t)bits);
    if ((lig & 1) == 0) stream_store(block_words + (lig >> 1), (uint32_t)bits | (nxt << 16));
  } else if constexpr (NB == 24) {
    // 4 lanes make 3 dwords: lane j < 3 of the quad stores (p_j >> 8j) | (p_{j+1} << (24 - 8j))
    uint32_t nxt = dpp<DPP_ROW_SHL1>((uint32_t)bits);
    int j = lig & 3;
    uint32_t d = ((uint32_t)bits >> (8 * j)) | (nxt << (24 - 8 * j));
    if (j < 3) stream_store(block_words + (lig >> 2) * 3 + j, d);
  } else if constexpr (NB == 48) {
    // 2 lanes make 3 dwords: even lane stores dwords 0 and 1, odd lane dword 2
    uint32_t nxt = dpp<DPP_ROW_SHL1>((uint32_t)bits);
    uint32_t* p = block_words + (lig >> 1) * 3;
    if ((lig & 1) == 0) {
      stream_store(p, (uint32_t)bits);
      stream_store(p + 1, (uint32_t)(bits >> 32) | (nxt << 16));
    } else {
      stream_store(p + 2, (uint32_t)(bits >> 16));
    }
  } else {
    static_assert(NB == 64, "odd element widths take the byte-staged path");
  }
}

constexpr bool direct_code_store(int nb) { return nb == 64 || nb == 32 || nb == 16 || nb == 24 || nb == 48; }

// Block sizes other than 32 (KG): the codes of a row are one bit string whatever the block size, so they are packed
// and stored in windows of 32 codes exactly as for k = 32; only the lanes that share a maximum, and the index of the
// scale byte, follow the block size (2^log2_lanes lanes of N elements).
template <int ELEM, bool HW, int DT, int U, int TPB, bool KG>
__global__ __launch_bounds__(TPB) void quantize_rows_kernel(const void* __restrict__ src, uint32_t* __restrict__ codes,
                                                            uint8_t* __restrict__ scales, int64_t nchunks,
                                                            uint32_t chunks_per_row, int64_t ld, int flat, int tie,
                                                            int log2_lanes) {
  using E = Elem<ELEM>;
  constexpr int N = Dense<DT>::N, G = 32 / N, W = E::bits;
  __shared__ uint32_t stage[direct_code_store(N * W) ? 1 : TPB * U * (N / 4)];
  int tid = threadIdx.x;
  if constexpr (HW && E::hw == HW_FP8) tid = set_fp8_saturation(tid);
  int64_t q0 = (int64_t)blockIdx.x * (TPB * U) + tid;
  // bf16 tensor and a 6-bit minifloat with a hardware conversion: the 8 bf16 values of a chunk are converted as they
  // were loaded (one 32-wide conversion whose other 24 inputs are zeros), and |V| is maximised on the 16-bit halves
  constexpr bool RAW6 = HW && DT == MX_BF16 && (E::hw == HW_FP6 || E::hw == HW_BF6);
  float v[U][N];
  u32x4 raw[U];
  bool live[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t q = q0 + TPB * u;
    live[u] = q < nchunks;
    if constexpr (RAW6) {
      raw[u] = u32x4{0u, 0u, 0u, 0u};
      if (live[u]) raw[u] = stream_load(reinterpret_cast<const u32x4*>(static_cast<const char*>(src) + chunk_offset<N>(q, chunks_per_row, ld, flat) * 2));
    } else {
      if (live[u]) load_chunk<DT>(src, chunk_offset<N>(q, chunks_per_row, ld, flat), v[u]);
      else {
#pragma unroll
        for (int i = 0; i < N; ++i) v[u][i] = 0.0f;
      }
    }
  }
  const int lig = tid & (G - 1);                                  // lane inside its window of 32 codes
  const int lane_in_block = KG ? (tid & ((1 << log2_lanes) - 1)) : lig;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t q = q0 + TPB * u;
    uint32_t byte;
    uint64_t bits;
    if constexpr (RAW6) {
      typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
      u16x2 m0 = __builtin_bit_cast(u16x2, raw[u].x & 0x7FFF7FFFu), m1 = __builtin_bit_cast(u16x2, raw[u].y & 0x7FFF7FFFu);
      u16x2 m2 = __builtin_bit_cast(u16x2, raw[u].z & 0x7FFF7FFFu), m3 = __builtin_bit_cast(u16x2, raw[u].w & 0x7FFF7FFFu);
      u16x2 m = __builtin_elementwise_max(__builtin_elementwise_max(m0, m1), __builtin_elementwise_max(m2, m3));
      uint32_t amax = (uint32_t)(m.x > m.y ? m.x : m.y) << 16;   // the fp32 bit pattern of the largest |V|
      byte = scale_byte_from_amax<E::emax>(block_max<G, KG>(amax, log2_lanes));
      u32x16 a = {raw[u].x, raw[u].y, raw[u].z, raw[u].w, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
      u32x6 p = cvt_pk32_fp6_bf16<E::hw == HW_BF6>(a, scale_operand(byte));
      bits = byte == 255u ? 0ull : ((uint64_t)p[0] | ((uint64_t)(p[1] & 0xFFFFu) << 32));
    } else {
      byte = scale_byte_from_amax<E::emax>(block_max<G, KG>(chunk_amax_bits(v[u]), log2_lanes));
      bits = byte == 255u ? 0ull : encode_chunk<ELEM, HW, N, DT == MX_BF16>(v[u], byte, tie);
    }
    int64_t blk = q / G;  // windows of 32 codes are numbered like the chunks: row-major
    if constexpr (direct_code_store(N * W)) {
      // a window's lanes are all live or all not (chunks per row is a multiple of the group size)
      if (live[u]) store_chunk_codes<W, N>(codes + blk * W, bits, lig);
    } else {
      // odd widths: stage one byte per code, repack one block per lane below
      uint32_t b4[N / 4];
#pragma unroll
      for (int i = 0; i < N / 4; ++i) {
        uint32_t r = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) r |= (uint32_t)((bits >> ((4 * i + k) * W)) & ((1u << W) - 1u)) << (8 * k);
        b4[i] = r;
      }
#pragma unroll
      for (int i = 0; i < N / 4; ++i) stage[(u * TPB + tid) * (N / 4) + i] = b4[i];
    }
    if (live[u] && lane_in_block == 0) scales[KG ? (q >> log2_lanes) : blk] = (uint8_t)byte;
  }
  if constexpr (!direct_code_store(N * W)) {
    __syncthreads();
    // TPB * U chunks = TPB * U / G blocks staged as 32 bytes each, in chunk order
    constexpr int BLOCKS = TPB * U / G;
    for (int b = tid; b < BLOCKS; b += TPB) {
      // chunk order inside the stage: u-major, then lane; block b of slab u' covers lanes [G*b', G*b'+G)
      int u2 = b / (TPB / G), bl = b % (TPB / G);
      int64_t blk = ((int64_t)blockIdx.x * (TPB * U) + TPB * u2) / G + bl;
      if (blk * G < nchunks) {
        uint32_t in[8], out[W];
#pragma unroll
        for (int i = 0; i < 8; ++i) in[i] = stage[(u2 * TPB + bl * G) * (N / 4) + i];
        pack_block_bytes<W>(in, out);
        store_dwords<W>(codes + blk * W, out);
      }
    }
  }
}

// ------------------------------------------------------------------ axis 1: dequantize
// N * W code bits of this lane's chunk out of the block's W dwords, with as few loads as the
// width allows (the lanes of a block read neighbouring or the same dwords).
template <int W, int N>
__device__ __forceinline__ uint64_t load_chunk_codes(const uint32_t* block_words, int lig) {
  constexpr int NB = N * W;
  if constexpr (NB == 64) {
    u32x2 t = stream_load(reinterpret_cast<const u32x2*>(block_words + 2 * lig));
    return (uint64_t)t.x | ((uint64_t)t.y << 32);
  } else if constexpr (NB == 32) {
    return block_words[lig];
  } else if constexpr (NB == 16) {
    return (block_words[lig >> 1] >> (16 * (lig & 1))) & 0xFFFFu;
  } else {
    int o = lig * NB, d = o >> 5, sh = o & 31;
    uint32_t w0 = block_words[d];
    uint32_t w1 = block_words[d + 1 < W ? d + 1 : W - 1];
    uint64_t r = ((uint64_t)w0 | ((uint64_t)w1 << 32)) >> sh;
    if constexpr (NB > 48) {  // a 56-bit piece can straddle three dwords
      uint32_t w2 = block_words[d + 2 < W ? d + 2 : W - 1];
      if (sh) r |= (uint64_t)w2 << (64 - sh);
    }
    return r & ((1ull << NB) - 1ull);
  }
}

template <int ELEM, int DT, int U, int TPB, bool KG>
__global__ __launch_bounds__(TPB) void dequant_rows_kernel(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                           void* __restrict__ dst, int64_t nchunks, uint32_t chunks_per_row,
                                                           int64_t ld, int flat, int log2_lanes) {
  using E = Elem<ELEM>;
  constexpr int N = Dense<DT>::N, G = 32 / N, W = E::bits;
  constexpr bool HW = E::hw != HW_NONE;
  int tid = threadIdx.x;
  int64_t q0 = (int64_t)blockIdx.x * (TPB * U) + tid;
  const int lig = tid & (G - 1);
  uint64_t bits[U];
  uint32_t byte[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t q = q0 + TPB * u;
    bits[u] = 0; byte[u] = 0;
    if (q < nchunks) {
      int64_t blk = q / G;   // window of 32 codes
      bits[u] = load_chunk_codes<W, N>(codes + blk * W, lig);
      byte[u] = scales[KG ? (q >> log2_lanes) : blk];
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t q = q0 + TPB * u;
    if (q < nchunks) {
      if constexpr (DT == MX_BF16 && (E::hw == HW_FP6 || E::hw == HW_BF6)) {
        // 6-bit minifloat codes straight to bf16: one conversion instruction for the lane's 8 codes (the other 24
        // inputs are zeros), its first 4 result dwords are the 16-byte output chunk
        u32x6 a = {(uint32_t)bits[u], (uint32_t)(bits[u] >> 32), 0u, 0u, 0u, 0u};
        u32x16 r = cvt_pk32_bf16_fp6<E::hw == HW_BF6>(a, scale_operand(byte[u]));
        u32x4 t = {r[0], r[1], r[2], r[3]};
        if (byte[u] == 255u) t = u32x4{0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u};
        stream_store(reinterpret_cast<u32x4*>(static_cast<char*>(dst) + chunk_offset<N>(q, chunks_per_row, ld, flat) * 2), t);
      } else {
        float v[N];
        decode_chunk<ELEM, HW, N>(bits[u], byte[u], v);
        if (byte[u] == 255u) {
#pragma unroll
          for (int i = 0; i < N; ++i) v[i] = __uint_as_float(0x7FC00000u);
        }
        store_chunk<DT>(dst, chunk_offset<N>(q, chunks_per_row, ld, flat), v);
      }
    }
  }
}

// ------------------------------------------------------------------ fake-quant of one chunk / column piece
// v (N elements of a block whose scale byte(s) are given) -> DQ(Q(v)) in place.
template <int TARGET, int ANCHOR, bool HW, int N, bool NARROW = false>
__device__ __forceinline__ void fake_quant_chunk(float (&v)[N], uint32_t byte_first, int tie) {
  // byte_first: scale byte of the format quantized first (the anchor if there is one)
  if (byte_first == 255u) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = __uint_as_float(0x7FC00000u);
    return;
  }
  if constexpr (ANCHOR < 0) {
    if constexpr (Elem<TARGET>::is_int && NARROW) {
      if (tie != MX_ROUND_HALF_EVEN) {
        // bf16 source, MXINT target: Round in one fma (see round_int_narrow), and X * P without going through codes
        const float scale = ldexpf(1.0f, 127 - (int)byte_first), x = ldexpf(1.0f, (int)byte_first - 127);
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = (float)round_int_narrow<Elem<TARGET>::bits>(v[i], scale) * x;
        return;
      }
    }
    uint64_t c = encode_chunk<TARGET, HW, N, NARROW>(v, byte_first, tie);
    decode_chunk<TARGET, HW, N>(c, byte_first, v);
  } else if constexpr (Elem<ANCHOR>::is_int) {
    // Eq. (7) with Eq. (4), all in integer registers: P_h = clip(Round(V / X_h)); P_l = clip(Round(P_h / 2^De)) is
    // (P_h + h - [P_h < 0]) >> De for half-away-from-zero and (P_h + h - 1 + bit_De(P_h)) >> De for half-to-even
    // (arithmetic shifts, h = 2^(De-1)); W_t = P_l * X_h * 2^De.
    constexpr int BH = Elem<ANCHOR>::bits, BL = Elem<TARGET>::bits, DE = BH - BL;
    constexpr int HALF = 1 << (DE - 1), LIM = (1 << (BL - 1)) - 1;
    int sh = 127 - (int)byte_first;
    uint32_t byte_l = byte_first + DE > 254u ? 254u : byte_first + DE;
    const float scale_h = ldexpf(1.0f, sh);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      int ph;
      if (NARROW && tie != MX_ROUND_HALF_EVEN) ph = round_int_narrow<BH>(v[i], scale_h);
      else ph = ((int)(encode_int_scaled<BH>(v[i], sh, tie) << (32 - BH))) >> (32 - BH);
      int pl = (tie == MX_ROUND_HALF_EVEN) ? (ph + (HALF - 1) + ((ph >> DE) & 1)) >> DE : (ph + HALF + (ph >> 31)) >> DE;
      pl = pl < -LIM ? -LIM : (pl > LIM ? LIM : pl);
      v[i] = ldexpf((float)pl, (int)byte_l - 127);
    }
  } else {
    // Eq. (7): W_A = Q_A(W); W_t = Q_{A->t}(W_A) = quantize_t(P_h / 2^De) with X_l = X_h 2^De
    constexpr int DE = Elem<ANCHOR>::emax - Elem<TARGET>::emax;
    uint64_t ch = encode_chunk<ANCHOR, HW, N>(v, byte_first, tie);
    float ph[N];
    decode_chunk<ANCHOR, HW, N>(ch, 127u, ph);               // the anchor elements P_h as numbers
    uint64_t cl = encode_chunk<TARGET, HW, N>(ph, 127u + DE, tie);
    uint32_t byte_l = byte_first + DE > 254u ? 254u : byte_first + DE;
    decode_chunk<TARGET, HW, N>(cl, byte_l, v);
  }
}

template <int TARGET, int ANCHOR>
struct FirstFormat { static constexpr int elem = ANCHOR < 0 ? TARGET : ANCHOR; };

template <int TARGET, int ANCHOR, bool HW, int DT, int U, int TPB, bool KG>
__global__ __launch_bounds__(TPB) void fake_quant_rows_kernel(const void* __restrict__ src, void* __restrict__ dst,
                                                              int64_t nchunks, uint32_t chunks_per_row, int64_t ld_src,
                                                              int64_t ld_dst, int flat_src, int flat_dst, int tie,
                                                              int log2_lanes) {
  constexpr int FIRST = FirstFormat<TARGET, ANCHOR>::elem;
  constexpr int N = Dense<DT>::N, G = 32 / N;
  int tid = threadIdx.x;
  if constexpr (HW && Elem<FIRST>::hw == HW_FP8) tid = set_fp8_saturation(tid);
  int64_t q0 = (int64_t)blockIdx.x * (TPB * U) + tid;
  float v[U][N];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t q = q0 + TPB * u;
    if (q < nchunks) load_chunk<DT>(src, chunk_offset<N>(q, chunks_per_row, ld_src, flat_src), v[u]);
    else {
#pragma unroll
      for (int i = 0; i < N; ++i) v[u][i] = 0.0f;
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t q = q0 + TPB * u;
    uint32_t byte = scale_byte_from_amax<Elem<FIRST>::emax>(block_max<G, KG>(chunk_amax_bits(v[u]), log2_lanes));
    using T = Elem<TARGET>;
    if constexpr (HW && DT == MX_BF16 && (T::hw == HW_FP6 || T::hw == HW_BF6) && (ANCHOR < 0 || !Elem<FIRST>::is_int)) {
      // 6-bit minifloat target, bf16 tensor: the codes go back to bf16 with one hardware conversion (exact for every
      // code and scale byte) instead of eight software decodes and four packs
      uint64_t c;
      uint32_t byte_t = byte;
      if constexpr (ANCHOR < 0) {
        c = encode_chunk<TARGET, HW, N>(v[u], byte, tie);
      } else {
        constexpr int DE = Elem<ANCHOR>::emax - T::emax;   // Eq. (7) through the MXFP8 anchor
        uint64_t ch = encode_chunk<ANCHOR, HW, N>(v[u], byte, tie);
        float ph[N];
        decode_chunk<ANCHOR, HW, N>(ch, 127u, ph);
        c = encode_chunk<TARGET, HW, N>(ph, 127u + DE, tie);
        byte_t = byte + DE > 254u ? 254u : byte + DE;
      }
      u32x6 a = {(uint32_t)c, (uint32_t)(c >> 32), 0u, 0u, 0u, 0u};
      u32x16 r = cvt_pk32_bf16_fp6<T::hw == HW_BF6>(a, scale_operand(byte_t));
      u32x4 t = {r[0], r[1], r[2], r[3]};
      if (byte == 255u) t = u32x4{0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u};
      if (q < nchunks)
        stream_store(reinterpret_cast<u32x4*>(static_cast<char*>(dst) + chunk_offset<N>(q, chunks_per_row, ld_dst, flat_dst) * 2), t);
    } else {
      fake_quant_chunk<TARGET, ANCHOR, HW, N, DT == MX_BF16>(v[u], byte, tie);
      if (q < nchunks) store_chunk<DT>(dst, chunk_offset<N>(q, chunks_per_row, ld_dst, flat_dst), v[u]);
    }
  }
}

// ------------------------------------------------------------------ axis 0 (blocks down a column)
// Work item = (row block rb, column quad cq): 4 adjacent columns x 32 rows in registers.
struct ColItem { int64_t rb; uint32_t cq; };
__device__ __forceinline__ ColItem col_item(int64_t item, uint32_t quads_per_row) {
  uint32_t rb = (uint32_t)((uint64_t)item / quads_per_row);
  return ColItem{(int64_t)rb, (uint32_t)((uint64_t)item - (uint64_t)rb * quads_per_row)};
}

template <int FIRST_EMAX>
__device__ __forceinline__ void column_bytes(const float (&v)[32][4], uint32_t (&byte)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t m = 0;
#pragma unroll
    for (int r = 0; r < 32; ++r) { uint32_t a = abs_bits(v[r][j]); m = m > a ? m : a; }
    byte[j] = scale_byte_from_amax<FIRST_EMAX>(m);
  }
}

// insert `nbits` bits at bit position `pos` (compile-time) of a W-dword string
template <int W, int POS, int NBITS>
__device__ __forceinline__ void insert_bits(uint32_t (&out)[W], uint64_t bits) {
  constexpr int d = POS >> 5, s = POS & 31;
  out[d] |= (uint32_t)(bits << s);
  if constexpr (s + NBITS > 32) out[d + 1] |= (uint32_t)(bits >> (32 - s));
  if constexpr (s + NBITS > 64) out[d + 2] |= (uint32_t)(bits >> (64 - s));
}
template <int W, int POS, int NBITS>
__device__ __forceinline__ uint64_t extract_bits(const uint32_t (&in)[W]) {
  constexpr int d = POS >> 5, s = POS & 31;
  uint64_t r = (uint64_t)in[d] >> s;
  if constexpr (s + NBITS > 32) r |= (uint64_t)in[d + 1] << (32 - s);
  if constexpr (s + NBITS > 64) r |= (uint64_t)in[d + 2] << (64 - s);
  if constexpr (NBITS < 64) r &= (1ull << NBITS) - 1ull;
  return r;
}

// The packed tensor of a column-blocked matrix is stored transposed ([cols][row blocks][W dwords]):
// a workgroup of RBS waves takes a tile of RBS consecutive row blocks x 256 columns (wave w = row block
// w, lane l = columns 4l..4l+3) and passes the codes through LDS, so that global memory sees, per
// column, the RBS * W contiguous dwords of its blocks instead of one isolated block per lane.  Runs
// shorter than 128 bytes per column cost a fifth of the bandwidth, so 4-bit and narrower formats take
// 8 row blocks per workgroup where the registers allow it.
// LDS layout: word[(rb_local * W + i) * 256 + col] -- a lane's 4 columns are one 128-bit access.
constexpr int kColTileCols = 256, kColTileRbs = 4;

template <int W, int RBS = kColTileRbs>
struct ColChunk {  // dwords per global access of the transposed side, by the alignment W guarantees
  static constexpr int cd = (W % 4 == 0) ? 4 : ((W % 2 == 0) ? 2 : 1);
  static constexpr int per_col = RBS * W / cd;
};

struct ColTile { int64_t rb0; int64_t c0; };
template <int RBS = kColTileRbs>
__device__ __forceinline__ ColTile col_tile(uint32_t col_groups) {
  uint32_t rbg = blockIdx.x / col_groups;
  return ColTile{(int64_t)rbg * RBS, (int64_t)(blockIdx.x - rbg * col_groups) * kColTileCols};
}

// The LDS tile <-> the transposed packed tensor: chunk k = (column k / PER_COL, part k % PER_COL) is CD consecutive
// dwords of that column's run of RBS * W dwords.  Plain accesses: a column's run is completed by several lanes, and L2
// merges them.  `valid_dw`: the dwords of the run that lie inside the tensor (a ragged last tile).
template <int W, int RBS, int TPB>
__device__ __forceinline__ void cols_tile_to_codes(const uint32_t* tile, uint32_t* __restrict__ codes, const ColTile& t, int64_t cols,
                                                   int64_t nrb, int valid_dw, int tid) {
  constexpr int CD = ColChunk<W, RBS>::cd, PER_COL = ColChunk<W, RBS>::per_col;
#pragma unroll
  for (int it = 0; it < kColTileCols * PER_COL / TPB; ++it) {
    int k = it * TPB + tid;
    int c = k / PER_COL, part = k - c * PER_COL;
    int d0 = part * CD;
    if (t.c0 + c < cols && d0 < valid_dw) {
      uint32_t w[CD];
#pragma unroll
      for (int q = 0; q < CD; ++q) w[q] = tile[(d0 + q) * kColTileCols + c];
      uint32_t* g = codes + ((t.c0 + c) * nrb + t.rb0) * W + d0;
      if (d0 + CD <= valid_dw) {
        store_dwords<CD>(g, w);
      } else {
#pragma unroll
        for (int q = 0; q < CD; ++q)
          if (d0 + q < valid_dw) g[q] = w[q];
      }
    }
  }
}
template <int W, int RBS, int TPB>
__device__ __forceinline__ void cols_codes_to_tile(uint32_t* tile, const uint32_t* __restrict__ codes, const ColTile& t, int64_t cols,
                                                   int64_t nrb, int valid_dw, int tid) {
  constexpr int CD = ColChunk<W, RBS>::cd, PER_COL = ColChunk<W, RBS>::per_col;
#pragma unroll
  for (int it = 0; it < kColTileCols * PER_COL / TPB; ++it) {
    int k = it * TPB + tid;
    int c = k / PER_COL, part = k - c * PER_COL;
    int d0 = part * CD;
    if (t.c0 + c < cols && d0 < valid_dw) {
      const uint32_t* g = codes + ((t.c0 + c) * nrb + t.rb0) * W + d0;
      uint32_t w[CD];
      if (d0 + CD <= valid_dw) {
        load_dwords<CD>(g, w);
      } else {
#pragma unroll
        for (int q = 0; q < CD; ++q) w[q] = d0 + q < valid_dw ? g[q] : 0u;
      }
#pragma unroll
      for (int q = 0; q < CD; ++q) tile[(d0 + q) * kColTileCols + c] = w[q];
    }
  }
}

// bf16 rows held as loaded (two columns per dword): largest |V| of each of the lane's 4 columns over its 32 rows, as
// fp32 bit patterns, from packed 16-bit maxima
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
template <int FIRST_EMAX>
__device__ __forceinline__ void column_bytes_bf16(const u32x2 (&raw)[32], uint32_t (&byte)[4]) {
  u16x2 m01 = {0, 0}, m23 = {0, 0};
#pragma unroll
  for (int r = 0; r < 32; ++r) {
    m01 = __builtin_elementwise_max(m01, __builtin_bit_cast(u16x2, raw[r].x & 0x7FFF7FFFu));
    m23 = __builtin_elementwise_max(m23, __builtin_bit_cast(u16x2, raw[r].y & 0x7FFF7FFFu));
  }
  byte[0] = scale_byte_from_amax<FIRST_EMAX>((uint32_t)m01.x << 16);
  byte[1] = scale_byte_from_amax<FIRST_EMAX>((uint32_t)m01.y << 16);
  byte[2] = scale_byte_from_amax<FIRST_EMAX>((uint32_t)m23.x << 16);
  byte[3] = scale_byte_from_amax<FIRST_EMAX>((uint32_t)m23.y << 16);
}

// RAW (bf16 tensors only): the 32 rows stay in registers as loaded, 64 instead of 128 registers, and are widened
// eight at a time when they are encoded.
template <int ELEM, bool HW, int DT, int RBS, bool RAW>
__global__ __launch_bounds__(64 * RBS) void quantize_cols_kernel(const void* __restrict__ src, uint32_t* __restrict__ codes,
                                                                 uint8_t* __restrict__ scales, int64_t cols, uint32_t col_groups,
                                                                 int64_t ld, int64_t nrb, int tie) {
  using E = Elem<ELEM>;
  static_assert(!RAW || DT == MX_BF16, "rows are kept as loaded only for bf16");
  constexpr int W = E::bits, TPB = 64 * RBS;
  __shared__ __attribute__((aligned(16))) uint32_t tile[RBS * W * kColTileCols];
  __shared__ __attribute__((aligned(8))) uint8_t tile_scales[kColTileCols * RBS];
  int tid = threadIdx.x;
  if constexpr (HW && E::hw == HW_FP8) tid = set_fp8_saturation(tid);
  const int wave = tid >> 6, lane = tid & 63;
  const ColTile t = col_tile<RBS>(col_groups);
  const int64_t rb = t.rb0 + wave, col = t.c0 + 4 * lane;
  if (rb < nrb && col < cols) {
    uint32_t byte[4];
    uint32_t out[4][W];
    if constexpr (RAW) {
      u32x2 raw[32];
      const char* p = static_cast<const char*>(src) + (rb * 32 * ld + col) * 2;
#pragma unroll
      for (int r = 0; r < 32; ++r) raw[r] = stream_load(reinterpret_cast<const u32x2*>(p + r * ld * 2));
      column_bytes_bf16<E::emax>(raw, byte);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int i = 0; i < W; ++i) out[j][i] = 0;
        static_for<0, 4>([&](auto cc) {
          constexpr int C = decltype(cc)::value;
          float x[8];
#pragma unroll
          for (int r = 0; r < 8; ++r) {
            uint32_t w = (j >> 1) ? raw[8 * C + r].y : raw[8 * C + r].x;
            x[r] = (j & 1) ? bf16_hi(w) : bf16_lo(w);
          }
          uint64_t bits = byte[j] == 255u ? 0ull : encode_chunk<ELEM, HW, 8, true>(x, byte[j], tie);
          insert_bits<W, C * 8 * W, 8 * W>(out[j], bits);
        });
      }
    } else {
      float v[32][4];
      int64_t off = rb * 32 * ld + col;
#pragma unroll
      for (int r = 0; r < 32; ++r) load_quad<DT>(src, off + r * ld, v[r]);
      column_bytes<E::emax>(v, byte);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int i = 0; i < W; ++i) out[j][i] = 0;
        static_for<0, 4>([&](auto cc) {
          constexpr int C = decltype(cc)::value;
          float x[8];
#pragma unroll
          for (int r = 0; r < 8; ++r) x[r] = v[8 * C + r][j];
          uint64_t bits = byte[j] == 255u ? 0ull : encode_chunk<ELEM, HW, 8, DT == MX_BF16>(x, byte[j], tie);
          insert_bits<W, C * 8 * W, 8 * W>(out[j], bits);
        });
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) tile_scales[(4 * lane + j) * RBS + wave] = (uint8_t)byte[j];
#pragma unroll
    for (int i = 0; i < W; ++i)
      *reinterpret_cast<u32x4*>(&tile[(wave * W + i) * kColTileCols + 4 * lane]) = u32x4{out[0][i], out[1][i], out[2][i], out[3][i]};
  }
  __syncthreads();
  const int64_t valid_rb = nrb - t.rb0 < RBS ? nrb - t.rb0 : RBS;
  const int valid_dw = (int)valid_rb * W;
  cols_tile_to_codes<W, RBS, TPB>(tile, codes, t, cols, nrb, valid_dw, tid);
  // scales: one column per thread, its (up to) RBS consecutive bytes
  if (tid < kColTileCols && t.c0 + tid < cols) {
    uint8_t* g = scales + (t.c0 + tid) * nrb + t.rb0;
    if (valid_rb == RBS && nrb % RBS == 0) {
      if constexpr (RBS == 8) *reinterpret_cast<u32x2*>(g) = *reinterpret_cast<const u32x2*>(&tile_scales[tid * RBS]);
      else *reinterpret_cast<uint32_t*>(g) = *reinterpret_cast<const uint32_t*>(&tile_scales[tid * RBS]);
    } else {
      for (int q = 0; q < (int)valid_rb; ++q) g[q] = tile_scales[tid * RBS + q];
    }
  }
}

// RBS row blocks per workgroup (one per wave): 4, or 8 for codes of 4 bits and fewer, whose runs per column would
// otherwise be 64 bytes and shorter.  (A kernel in which every lane fetched the 16 bytes of a 4-bit block itself, without
// the LDS pass, was faster while the packed tensor sat in the last-level cache -- 0.80 against 0.73 -- and slower when it
// came from HBM, 0.44 against 0.54: not kept.)
template <int ELEM, int DT, int RBS>
__global__ __launch_bounds__(64 * RBS) void dequant_cols_kernel(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                           void* __restrict__ dst, int64_t cols, uint32_t col_groups,
                                                           int64_t ld, int64_t nrb) {
  using E = Elem<ELEM>;
  constexpr int W = E::bits;
  constexpr bool HW = E::hw != HW_NONE;
  __shared__ __attribute__((aligned(16))) uint32_t tile[RBS * W * kColTileCols];
  __shared__ __attribute__((aligned(4))) uint8_t tile_scales[kColTileCols * RBS];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const ColTile t = col_tile<RBS>(col_groups);
  const int64_t valid_rb = nrb - t.rb0 < RBS ? nrb - t.rb0 : RBS;
  const int valid_dw = (int)valid_rb * W;
  cols_codes_to_tile<W, RBS, 64 * RBS>(tile, codes, t, cols, nrb, valid_dw, tid);
  if (tid < kColTileCols && t.c0 + tid < cols) {
    const uint8_t* g = scales + (t.c0 + tid) * nrb + t.rb0;
    for (int q = 0; q < (int)valid_rb; ++q) tile_scales[tid * RBS + q] = g[q];
  }
  __syncthreads();
  const int64_t rb = t.rb0 + wave, col = t.c0 + 4 * lane;
  if (rb < nrb && col < cols) {
    float v[32][4];
    uint32_t in[4][W];
#pragma unroll
    for (int i = 0; i < W; ++i) {
      u32x4 q = *reinterpret_cast<const u32x4*>(&tile[(wave * W + i) * kColTileCols + 4 * lane]);
      in[0][i] = q.x; in[1][i] = q.y; in[2][i] = q.z; in[3][i] = q.w;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t byte = tile_scales[(4 * lane + j) * RBS + wave];
      static_for<0, 4>([&](auto cc) {
        constexpr int C = decltype(cc)::value;
        float x[8];
        decode_chunk<ELEM, HW, 8>(extract_bits<W, C * 8 * W, 8 * W>(in[j]), byte, x);
#pragma unroll
        for (int r = 0; r < 8; ++r) v[8 * C + r][j] = byte == 255u ? __uint_as_float(0x7FC00000u) : x[r];
      });
    }
    int64_t off = rb * 32 * ld + col;
#pragma unroll
    for (int r = 0; r < 32; ++r) store_quad<DT>(dst, off + r * ld, v[r]);
  }
}

template <int TARGET, int ANCHOR, bool HW, int DT, int TPB>
__global__ __launch_bounds__(TPB) void fake_quant_cols_kernel(const void* __restrict__ src, void* __restrict__ dst,
                                                              int64_t nitems, uint32_t quads_per_row, int64_t ld_src,
                                                              int64_t ld_dst, int tie) {
  constexpr int FIRST = FirstFormat<TARGET, ANCHOR>::elem;
  int tid = threadIdx.x;
  if constexpr (HW && Elem<FIRST>::hw == HW_FP8) tid = set_fp8_saturation(tid);
  int64_t item = (int64_t)blockIdx.x * TPB + tid;
  if (item >= nitems) return;
  ColItem it = col_item(item, quads_per_row);
  float v[32][4];
  int64_t off = it.rb * 32 * ld_src + (int64_t)it.cq * 4;
#pragma unroll
  for (int r = 0; r < 32; ++r) load_quad<DT>(src, off + r * ld_src, v[r]);
  uint32_t byte[4];
  column_bytes<Elem<FIRST>::emax>(v, byte);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float x[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) x[r] = v[8 * c + r][j];
      fake_quant_chunk<TARGET, ANCHOR, HW, 8, DT == MX_BF16>(x, byte[j], tie);
#pragma unroll
      for (int r = 0; r < 8; ++r) v[8 * c + r][j] = x[r];
    }
  }
  int64_t offd = it.rb * 32 * ld_dst + (int64_t)it.cq * 4;
#pragma unroll
  for (int r = 0; r < 32; ++r) store_quad<DT>(dst, offd + r * ld_dst, v[r]);
}

// DQ(Q(.)) of a lane's R x N values (column j under scale byte `byte[j]`) for the 6-bit minifloats, whose hardware
// conversion takes 32 values under ONE scale: the values are first divided by their own column's scale (ldexp: exact,
// or so far below the smallest code that they round to zero either way) -- or, with an E4M3 anchor, replaced by their
// anchor elements P_h, which all share the scale 2^De of Eq. (6) -- then converted 32 at a time under one scale, and
// every code is read back under its column's scale (X P: exact, at most 4 significant bits).
template <int TARGET, int ANCHOR, int R, int N>
__device__ __forceinline__ void fake_quant_fp6_columns(float (&v)[R][N], const uint32_t (&byte)[N], int tie) {
  using E = Elem<TARGET>;
  constexpr int TOTAL = R * N, BATCHES = (TOTAL + 31) / 32;
  uint32_t byte_out[N];
  float s;
  if constexpr (ANCHOR < 0) {
#pragma unroll
    for (int j = 0; j < N; ++j) {
      byte_out[j] = byte[j];
#pragma unroll
      for (int r = 0; r < R; ++r) v[r][j] = ldexpf(v[r][j], 127 - (int)byte[j]);
    }
    s = scale_operand(127u);
  } else {
    constexpr int DE = Elem<ANCHOR>::emax - E::emax, PIECE = R < 8 ? R : 8;
#pragma unroll
    for (int j = 0; j < N; ++j) {
      byte_out[j] = byte[j] + DE > 254u ? 254u : byte[j] + DE;
#pragma unroll
      for (int c = 0; c < R / PIECE; ++c) {
        float x[PIECE];
#pragma unroll
        for (int r = 0; r < PIECE; ++r) x[r] = v[PIECE * c + r][j];
        uint64_t ch = encode_chunk<ANCHOR, true, PIECE>(x, byte[j], tie);
        decode_chunk<ANCHOR, true, PIECE>(ch, 127u, x);               // the anchor elements P_h as numbers
#pragma unroll
        for (int r = 0; r < PIECE; ++r) v[PIECE * c + r][j] = x[r];
      }
    }
    s = scale_operand(127u + DE);
  }
  static_for<0, BATCHES>([&](auto bc) {
    constexpr int B = decltype(bc)::value;
    f32x16 ev = {}, od = {};   // value e of the batch = flat element 32 B + e = v[(32 B + e) / N][(32 B + e) % N]
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int e0 = 32 * B + 2 * i, e1 = e0 + 1;
      if (e0 < TOTAL) ev[i] = v[e0 / N][e0 % N];
      if (e1 < TOTAL) od[i] = v[e1 / N][e1 % N];
    }
    const u32x6 p = cvt_2xpk16_fp6_f32<E::hw == HW_BF6>(ev, od, s);   // element 2i = ev[i], 2i + 1 = od[i]
    static_for<0, 32>([&](auto ec) {
      constexpr int EI = decltype(ec)::value, FLAT = 32 * B + EI;
      if constexpr (FLAT < TOTAL) {
        constexpr int POS = 6 * EI, W = POS / 32, SH = POS % 32;
        uint32_t c = p[W] >> SH;
        if constexpr (SH > 26) c |= p[W + 1] << (32 - SH);
        const uint32_t f = ((c & 0x1Fu) << (23 - E::mu)) | ((c & 0x20u) << 26);
        constexpr int J = FLAT % N;
        // (a minifloat without Inf / NaN in the top of an fp32's fields reads as its value times 2^(bias - 127))
        v[FLAT / N][J] = byte[J] == 255u ? __uint_as_float(0x7FC00000u)
                                         : ldexpf(__uint_as_float(f), (int)byte_out[J] - 127 + (127 - E::bias));
      }
    });
  });
}

// The same map with the rows of a block dealt to the waves of a workgroup (k = 32: eight waves of 4 rows; 64 and 128:
// eight waves of 8 and 16 rows; 16: four waves of 4): a wave loads its rows as 64 chunks of 16 bytes (1 KB per row),
// the waves exchange their columns' partial maxima through LDS (planes of dwords), and every wave converts and stores
// its own rows.  Four loads in flight per lane instead of 32 and a third of the registers: many small waves per compute
// unit, which is what a launch of well under 100 us needs to ramp up and drain quickly (32768 x 4096 bf16, k = 32: 0.79
// of the HBM peak against 0.75-0.76 for the 32-rows-per-lane kernel; on a tensor four times the size both stream at
// 0.81-0.82).  Needs the column count to be a multiple of the chunk (8 bf16 / 4 fp32 columns).
template <int TARGET, int ANCHOR, bool HW, int DT, int WAVES, int RPW>
__global__ __launch_bounds__(64 * WAVES) void fake_quant_cols_split_kernel(const void* __restrict__ src, void* __restrict__ dst,
                                                                           uint32_t chunks_per_row, uint32_t col_groups,
                                                                           int64_t ld_src, int64_t ld_dst, int tie) {
  constexpr int FIRST = FirstFormat<TARGET, ANCHOR>::elem;
  constexpr int N = Dense<DT>::N, PIECE = RPW < 8 ? RPW : 8;   // rows converted per call
  static_assert(RPW % PIECE == 0, "rows per wave");
  __shared__ uint32_t part[WAVES][N][64];
  int tid = threadIdx.x;
  if constexpr (HW && Elem<FIRST>::hw == HW_FP8) tid = set_fp8_saturation(tid);
  const int lane = tid & 63, wave = tid >> 6;
  const int64_t blk = (int64_t)(blockIdx.x / col_groups);
  const uint32_t chunk = (blockIdx.x % col_groups) * 64u + (uint32_t)lane;
  const bool live = chunk < chunks_per_row;   // (a lane past the row's end takes part in the barrier only)
  float v[RPW][N];
  const int64_t row0 = blk * (WAVES * RPW) + wave * RPW;
  if (live) {
#pragma unroll
    for (int r = 0; r < RPW; ++r) load_chunk<DT>(src, (row0 + r) * ld_src + (int64_t)chunk * N, v[r]);
  } else {
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
      for (int j = 0; j < N; ++j) v[r][j] = 0.f;
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    uint32_t m = 0;
#pragma unroll
    for (int r = 0; r < RPW; ++r) { uint32_t a = abs_bits(v[r][j]); m = m > a ? m : a; }
    part[wave][j][lane] = m;
  }
  __syncthreads();
  uint32_t byte[N];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    uint32_t m = part[0][j][lane];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) { uint32_t a = part[w][j][lane]; m = m > a ? m : a; }
    byte[j] = scale_byte_from_amax<Elem<FIRST>::emax>(m);
  }
  if constexpr (HW && (Elem<TARGET>::hw == HW_FP6 || Elem<TARGET>::hw == HW_BF6)) {
    fake_quant_fp6_columns<TARGET, ANCHOR, RPW, N>(v, byte, tie);
  } else {
#pragma unroll
    for (int j = 0; j < N; ++j) {
#pragma unroll
      for (int c = 0; c < RPW / PIECE; ++c) {
        float x[PIECE];
#pragma unroll
        for (int r = 0; r < PIECE; ++r) x[r] = v[PIECE * c + r][j];
        fake_quant_chunk<TARGET, ANCHOR, HW, PIECE, DT == MX_BF16>(x, byte[j], tie);
#pragma unroll
        for (int r = 0; r < PIECE; ++r) v[PIECE * c + r][j] = x[r];
      }
    }
  }
  if (live) {
#pragma unroll
    for (int r = 0; r < RPW; ++r) store_chunk<DT>(dst, (row0 + r) * ld_dst + (int64_t)chunk * N, v[r]);
  }
}

// ------------------------------------------------------------------ axis 0, blocks of 16, 64 or 128 rows
// The codes of a column are one bit string whatever the block size, so the packed tensor has the layout of k = 32 and
// these kernels keep its 32-row windows: a workgroup of 4 waves takes 4 consecutive windows x 256 columns (wave w =
// window w, lane l = columns 4l..4l+3).  What changes is which rows share a maximum and where the scale byte lives:
// k = 16: two scale bytes per window (rows 0-15 and 16-31); k = 64 / 128: the 2 / 4 windows of a block join their
// maxima through LDS (a block never straddles a workgroup: tiles start at multiples of 4 windows).  Scale bytes go
// straight to / come straight from global memory.  Plain kernels (rows widened to fp32, no packed-row variants): the
// benchmark's block is 32.
struct ColBlockGeom {
  int g;          // windows per block (k = 64: 2, k = 128: 4; k = 16: 1, with two blocks per window)
  int halves;     // blocks per window (k = 16: 2, else 1)
  int64_t nsb;    // scale bytes per column
};
__device__ __forceinline__ ColBlockGeom col_block_geom(int block, int64_t nrb) {
  if (block == 16) return ColBlockGeom{1, 2, 2 * nrb};
  const int g = block / 32;
  return ColBlockGeom{g, 1, nrb / g};
}
// scale-byte index of half h (rows 16 h ..) of window rb of a column
__device__ __forceinline__ int64_t col_block_scale_index(const ColBlockGeom& geo, int64_t rb, int h) {
  return geo.halves == 2 ? 2 * rb + h : rb / geo.g;
}

// largest |V| (fp32 bits) of each of the lane's 4 columns over the two halves of its window
__device__ __forceinline__ void column_half_amax(const float (&v)[32][4], uint32_t (&m)[4][2]) {
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t a = 0;
#pragma unroll
      for (int r = 0; r < 16; ++r) { uint32_t b = abs_bits(v[16 * h + r][j]); a = a > b ? a : b; }
      m[j][h] = a;
    }
}

// The scale bytes of the lane's 4 columns, per half of its window, from the half maxima: the blocks of 64 / 128 rows
// join the maxima of their windows through `xch` ([4 windows][256 columns]).  Every wave of the workgroup must call it.
template <int FIRST_EMAX>
__device__ __forceinline__ void column_block_bytes(const uint32_t (&m)[4][2], uint32_t (&byte)[4][2], const ColBlockGeom& geo,
                                                   uint32_t (*xch)[kColTileCols], int wave, int lane) {
  if (geo.halves == 2) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int h = 0; h < 2; ++h) byte[j][h] = scale_byte_from_amax<FIRST_EMAX>(m[j][h]);
    return;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) xch[wave][4 * lane + j] = m[j][0] > m[j][1] ? m[j][0] : m[j][1];
  __syncthreads();
  const int base = wave & ~(geo.g - 1);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t a = 0;
    for (int q = 0; q < geo.g; ++q) { uint32_t b = xch[base + q][4 * lane + j]; a = a > b ? a : b; }
    byte[j][0] = byte[j][1] = scale_byte_from_amax<FIRST_EMAX>(a);
  }
}

template <int ELEM, bool HW, int DT>
__global__ __launch_bounds__(256) void quantize_cols_kblock_kernel(const void* __restrict__ src, uint32_t* __restrict__ codes,
                                                                   uint8_t* __restrict__ scales, int64_t cols, uint32_t col_groups,
                                                                   int64_t ld, int64_t nrb, int tie, int block) {
  using E = Elem<ELEM>;
  constexpr int W = E::bits;
  __shared__ __attribute__((aligned(16))) uint32_t tile[kColTileRbs * W * kColTileCols];
  __shared__ uint32_t xch[kColTileRbs][kColTileCols];
  int tid = threadIdx.x;
  if constexpr (HW && E::hw == HW_FP8) tid = set_fp8_saturation(tid);
  const int wave = tid >> 6, lane = tid & 63;
  const ColTile t = col_tile(col_groups);
  const ColBlockGeom geo = col_block_geom(block, nrb);
  const int64_t rb = t.rb0 + wave, col = t.c0 + 4 * lane;
  const bool active = rb < nrb && col < cols;
  float v[32][4];
  if (active) {
    const int64_t off = rb * 32 * ld + col;
#pragma unroll
    for (int r = 0; r < 32; ++r) load_quad<DT>(src, off + r * ld, v[r]);
  } else {
#pragma unroll
    for (int r = 0; r < 32; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) v[r][j] = 0.0f;
  }
  uint32_t m[4][2], byte[4][2];
  column_half_amax(v, m);
  column_block_bytes<E::emax>(m, byte, geo, xch, wave, lane);
  if (active) {
    uint32_t out[4][W];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int i = 0; i < W; ++i) out[j][i] = 0;
      static_for<0, 4>([&](auto cc) {
        constexpr int C = decltype(cc)::value;
        float x[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) x[r] = v[8 * C + r][j];
        const uint32_t b = byte[j][C >> 1];
        uint64_t bits = b == 255u ? 0ull : encode_chunk<ELEM, HW, 8, DT == MX_BF16>(x, b, tie);
        insert_bits<W, C * 8 * W, 8 * W>(out[j], bits);
      });
      uint8_t* sc = scales + (col + j) * geo.nsb;
      if (geo.halves == 2) {
        sc[2 * rb] = (uint8_t)byte[j][0];
        sc[2 * rb + 1] = (uint8_t)byte[j][1];
      } else if ((wave & (geo.g - 1)) == 0) {
        sc[rb / geo.g] = (uint8_t)byte[j][0];
      }
    }
#pragma unroll
    for (int i = 0; i < W; ++i)
      *reinterpret_cast<u32x4*>(&tile[(wave * W + i) * kColTileCols + 4 * lane]) = u32x4{out[0][i], out[1][i], out[2][i], out[3][i]};
  }
  __syncthreads();
  const int64_t valid_rb = nrb - t.rb0 < kColTileRbs ? nrb - t.rb0 : kColTileRbs;
  const int valid_dw = (int)valid_rb * W;
  cols_tile_to_codes<W, kColTileRbs, 256>(tile, codes, t, cols, nrb, valid_dw, tid);
}

template <int ELEM, int DT>
__global__ __launch_bounds__(256) void dequant_cols_kblock_kernel(const uint32_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                                  void* __restrict__ dst, int64_t cols, uint32_t col_groups,
                                                                  int64_t ld, int64_t nrb, int block) {
  using E = Elem<ELEM>;
  constexpr int W = E::bits;
  constexpr bool HW = E::hw != HW_NONE;
  __shared__ __attribute__((aligned(16))) uint32_t tile[kColTileRbs * W * kColTileCols];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const ColTile t = col_tile(col_groups);
  const ColBlockGeom geo = col_block_geom(block, nrb);
  const int64_t valid_rb = nrb - t.rb0 < kColTileRbs ? nrb - t.rb0 : kColTileRbs;
  const int valid_dw = (int)valid_rb * W;
  cols_codes_to_tile<W, kColTileRbs, 256>(tile, codes, t, cols, nrb, valid_dw, tid);
  __syncthreads();
  const int64_t rb = t.rb0 + wave, col = t.c0 + 4 * lane;
  if (rb < nrb && col < cols) {
    float v[32][4];
    uint32_t in[4][W];
#pragma unroll
    for (int i = 0; i < W; ++i) {
      u32x4 q = *reinterpret_cast<const u32x4*>(&tile[(wave * W + i) * kColTileCols + 4 * lane]);
      in[0][i] = q.x; in[1][i] = q.y; in[2][i] = q.z; in[3][i] = q.w;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint8_t* sc = scales + (col + j) * geo.nsb;
      const uint32_t b0 = sc[col_block_scale_index(geo, rb, 0)], b1 = sc[col_block_scale_index(geo, rb, 1)];
      static_for<0, 4>([&](auto cc) {
        constexpr int C = decltype(cc)::value;
        const uint32_t byte = (C >> 1) ? b1 : b0;
        float x[8];
        decode_chunk<ELEM, HW, 8>(extract_bits<W, C * 8 * W, 8 * W>(in[j]), byte, x);
#pragma unroll
        for (int r = 0; r < 8; ++r) v[8 * C + r][j] = byte == 255u ? __uint_as_float(0x7FC00000u) : x[r];
      });
    }
    int64_t off = rb * 32 * ld + col;
#pragma unroll
    for (int r = 0; r < 32; ++r) store_quad<DT>(dst, off + r * ld, v[r]);
  }
}

template <int TARGET, int ANCHOR, bool HW, int DT>
__global__ __launch_bounds__(256) void fake_quant_cols_kblock_kernel(const void* __restrict__ src, void* __restrict__ dst,
                                                                     int64_t cols, uint32_t col_groups, int64_t ld_src,
                                                                     int64_t ld_dst, int64_t nrb, int tie, int block) {
  constexpr int FIRST = FirstFormat<TARGET, ANCHOR>::elem;
  __shared__ uint32_t xch[kColTileRbs][kColTileCols];
  int tid = threadIdx.x;
  if constexpr (HW && Elem<FIRST>::hw == HW_FP8) tid = set_fp8_saturation(tid);
  const int wave = tid >> 6, lane = tid & 63;
  const ColTile t = col_tile(col_groups);
  const ColBlockGeom geo = col_block_geom(block, nrb);
  const int64_t rb = t.rb0 + wave, col = t.c0 + 4 * lane;
  const bool active = rb < nrb && col < cols;
  float v[32][4];
  if (active) {
    const int64_t off = rb * 32 * ld_src + col;
#pragma unroll
    for (int r = 0; r < 32; ++r) load_quad<DT>(src, off + r * ld_src, v[r]);
  } else {
#pragma unroll
    for (int r = 0; r < 32; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) v[r][j] = 0.0f;
  }
  uint32_t m[4][2], byte[4][2];
  column_half_amax(v, m);
  column_block_bytes<Elem<FIRST>::emax>(m, byte, geo, xch, wave, lane);
  if (!active) return;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float x[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) x[r] = v[8 * c + r][j];
      fake_quant_chunk<TARGET, ANCHOR, HW, 8, DT == MX_BF16>(x, byte[j][c >> 1], tie);
#pragma unroll
      for (int r = 0; r < 8; ++r) v[8 * c + r][j] = x[r];
    }
  }
  const int64_t offd = rb * 32 * ld_dst + col;
#pragma unroll
  for (int r = 0; r < 32; ++r) store_quad<DT>(dst, offd + r * ld_dst, v[r]);
}

// ------------------------------------------------------------------ host launchers
// Launch shape of the row-axis kernels: chunks per lane and lanes per workgroup.  Which shape streams best
// depends on the read : write mix and on the arithmetic per element, so it is chosen per element format
// (measured on 1 GiB bf16 tensors; the figures are percent of the 8 TB/s HBM peak).
struct RowsShape { int unroll, threads; };
template <int ELEM>
constexpr RowsShape quantize_shape() {
  using E = Elem<ELEM>;
  if (E::is_int) return RowsShape{4, 64};                                      // MXINT8 / 6 / 4: 82 / 79 / 82 (1 x 64: 70 - 75)
  if (E::hw == HW_FP8) return RowsShape{2, 128};                               // 83
  if (E::hw != HW_NONE) return RowsShape{2, 64};                               // E2M1 85 (1 x 64: 73), FP6 79
  return RowsShape{1, 256};
}
template <int ELEM, int DT>
constexpr RowsShape dequant_shape() {
  using E = Elem<ELEM>;
  if (DT == MX_F32) {   // 4 elements per lane: half the code bytes per load of the bf16 case (16384 x 28672 tensor)
    if (E::bits == 8) return RowsShape{2, 128};                                // 84 (1 x 64: 65)
    if (E::bits == 4 && !E::is_int) return RowsShape{1, 256};                  // 92 (2 x 256: 87)
  }
  if (E::bits == 4) return E::is_int ? RowsShape{4, 256} : RowsShape{2, 256};  // 79, 83 (1 x 64: 63, 65)
  if (E::bits == 6) return RowsShape{1, 256};                                  // FP6 79 (one conversion per lane), MXINT6 73
  return RowsShape{1, 64};                                                     // 8-bit: 83
}
constexpr int kFqUnroll = 1;                  // fake-quant: one chunk per lane, one wave per workgroup (82 - 83)
constexpr int kFqThreads = 64;


// lanes of N elements per block of `block` elements, as a power of two (block = 16 .. 128, N = 4 or 8)
static inline int log2_lanes_of(int block, int n) {
  int lanes = block / n, l = 0;
  while ((1 << l) < lanes) ++l;
  return l;
}

template <int ELEM, bool HW, int DT>
static mx_status_t run_quantize(int axis, int block, int tie, const DenseArg& s, void* codes, uint8_t* scales, hipStream_t st) {
  if (axis == 1) {
    constexpr int N = Dense<DT>::N;
    int64_t cpr = s.cols / N, nchunks = s.rows * cpr;
    if (cpr > 0xFFFFFFFFll) return MX_ERR_UNSUPPORTED;
    constexpr RowsShape shape = quantize_shape<ELEM>();
    int64_t wgs = (nchunks + shape.threads * shape.unroll - 1) / (shape.threads * shape.unroll);
    if (wgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    if (block == 32)
      hipLaunchKernelGGL((quantize_rows_kernel<ELEM, HW, DT, shape.unroll, shape.threads, false>), dim3((unsigned)wgs), dim3(shape.threads), 0, st,
                         s.data, static_cast<uint32_t*>(codes), scales, nchunks, (uint32_t)cpr, s.ld, (int)(s.ld == s.cols), tie, 0);
    else
      hipLaunchKernelGGL((quantize_rows_kernel<ELEM, HW, DT, shape.unroll, shape.threads, true>), dim3((unsigned)wgs), dim3(shape.threads), 0, st,
                         s.data, static_cast<uint32_t*>(codes), scales, nchunks, (uint32_t)cpr, s.ld, (int)(s.ld == s.cols), tie,
                         log2_lanes_of(block, N));
  } else if (block != 32) {
    if (s.cols % 4 || s.rows % 32) return MX_ERR_UNSUPPORTED;
    const int64_t nrb = s.rows / 32, cgs = (s.cols + kColTileCols - 1) / kColTileCols, rbgs = (nrb + kColTileRbs - 1) / kColTileRbs;
    if (cgs * rbgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((quantize_cols_kblock_kernel<ELEM, HW, DT>), dim3((unsigned)(cgs * rbgs)), dim3(256), 0, st, s.data,
                       static_cast<uint32_t*>(codes), scales, s.cols, (uint32_t)cgs, s.ld, nrb, tie, block);
  } else {
    if (s.cols % 4) return MX_ERR_UNSUPPORTED;
    int64_t nrb = s.rows / 32;
    // bf16 rows stay packed in registers where that pays (measured on 32768 x 4096): the 4-bit and narrower formats,
    // which then afford 8 row blocks per workgroup (128-byte runs per column: 62 -> 70 % of HBM peak), and the 6-bit
    // minifloats, whose 32-wide conversions otherwise need 288 registers (41 -> 63 %)
    using E = Elem<ELEM>;
    constexpr bool RAW = DT == MX_BF16 && (E::bits <= 4 || (HW && (E::hw == HW_FP6 || E::hw == HW_BF6)));
    constexpr int RBS = (RAW && E::bits <= 4) ? 8 : kColTileRbs;
    int64_t cgs = (s.cols + kColTileCols - 1) / kColTileCols, rbgs = (nrb + RBS - 1) / RBS;
    if (cgs * rbgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((quantize_cols_kernel<ELEM, HW, DT, RBS, RAW>), dim3((unsigned)(cgs * rbgs)), dim3(64 * RBS), 0, st, s.data,
                       static_cast<uint32_t*>(codes), scales, s.cols, (uint32_t)cgs, s.ld, nrb, tie);
  }
  return launch_status("a dense kernel");
}

template <int ELEM, int DT>
static mx_status_t run_dequant(int axis, int block, const void* codes, const uint8_t* scales, const DenseArg& d, hipStream_t st) {
  if (axis == 1) {
    constexpr int N = Dense<DT>::N;
    int64_t cpr = d.cols / N, nchunks = d.rows * cpr;
    if (cpr > 0xFFFFFFFFll) return MX_ERR_UNSUPPORTED;
    constexpr RowsShape shape = dequant_shape<ELEM, DT>();
    int64_t wgs = (nchunks + shape.threads * shape.unroll - 1) / (shape.threads * shape.unroll);
    if (wgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    if (block == 32)
      hipLaunchKernelGGL((dequant_rows_kernel<ELEM, DT, shape.unroll, shape.threads, false>), dim3((unsigned)wgs), dim3(shape.threads), 0, st,
                         static_cast<const uint32_t*>(codes), scales, d.data, nchunks, (uint32_t)cpr, d.ld, (int)(d.ld == d.cols), 0);
    else
      hipLaunchKernelGGL((dequant_rows_kernel<ELEM, DT, shape.unroll, shape.threads, true>), dim3((unsigned)wgs), dim3(shape.threads), 0, st,
                         static_cast<const uint32_t*>(codes), scales, d.data, nchunks, (uint32_t)cpr, d.ld, (int)(d.ld == d.cols),
                         log2_lanes_of(block, N));
  } else if (block != 32) {
    if (d.cols % 4 || d.rows % 32) return MX_ERR_UNSUPPORTED;
    const int64_t nrb = d.rows / 32, cgs = (d.cols + kColTileCols - 1) / kColTileCols, rbgs = (nrb + kColTileRbs - 1) / kColTileRbs;
    if (cgs * rbgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((dequant_cols_kblock_kernel<ELEM, DT>), dim3((unsigned)(cgs * rbgs)), dim3(256), 0, st,
                       static_cast<const uint32_t*>(codes), scales, d.data, d.cols, (uint32_t)cgs, d.ld, nrb, block);
  } else {
    if (d.cols % 4) return MX_ERR_UNSUPPORTED;
    int64_t nrb = d.rows / 32;
    constexpr int RBS = Elem<ELEM>::bits <= 4 ? 8 : kColTileRbs;
    int64_t cgs = (d.cols + kColTileCols - 1) / kColTileCols, rbgs = (nrb + RBS - 1) / RBS;
    if (cgs * rbgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((dequant_cols_kernel<ELEM, DT, RBS>), dim3((unsigned)(cgs * rbgs)), dim3(64 * RBS), 0, st,
                       static_cast<const uint32_t*>(codes), scales, d.data, d.cols, (uint32_t)cgs, d.ld, nrb);
  }
  return launch_status("a dense kernel");
}

template <int TARGET, int ANCHOR, bool HW, int DT>
static mx_status_t run_fake_quant(int axis, int block, int tie, const DenseArg& s, const DenseArg& d, hipStream_t st) {
  if (axis == 1) {
    constexpr int N = Dense<DT>::N;
    int64_t cpr = s.cols / N, nchunks = s.rows * cpr;
    if (cpr > 0xFFFFFFFFll) return MX_ERR_UNSUPPORTED;
    int64_t wgs = (nchunks + kFqThreads * kFqUnroll - 1) / (kFqThreads * kFqUnroll);
    if (wgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    if (block == 32)
      hipLaunchKernelGGL((fake_quant_rows_kernel<TARGET, ANCHOR, HW, DT, kFqUnroll, kFqThreads, false>), dim3((unsigned)wgs), dim3(kFqThreads), 0,
                         st, s.data, d.data, nchunks, (uint32_t)cpr, s.ld, d.ld, (int)(s.ld == s.cols), (int)(d.ld == d.cols), tie, 0);
    else
      hipLaunchKernelGGL((fake_quant_rows_kernel<TARGET, ANCHOR, HW, DT, kFqUnroll, kFqThreads, true>), dim3((unsigned)wgs), dim3(kFqThreads), 0,
                         st, s.data, d.data, nchunks, (uint32_t)cpr, s.ld, d.ld, (int)(s.ld == s.cols), (int)(d.ld == d.cols), tie,
                         log2_lanes_of(block, N));
  } else if (s.cols % Dense<DT>::N == 0 && s.cols / Dense<DT>::N <= 0xFFFFFFFFll && s.rows % 32 == 0 &&
             (s.rows / block) * ((s.cols / Dense<DT>::N + 63) / 64) <= 0x7FFFFFFF) {
    // (the axis extent is a multiple of the block: checked at the boundary; and of 32 also for blocks of 16, as for the
    // packed tensors, so that one rule holds for all three operations whatever the column count)
    const int64_t cpr = s.cols / Dense<DT>::N, cgs = (cpr + 63) / 64, nblk = s.rows / block;
#define MX_FQ_SPLIT(WAVES, RPW)                                                                                          \
    hipLaunchKernelGGL((fake_quant_cols_split_kernel<TARGET, ANCHOR, HW, DT, WAVES, RPW>), dim3((unsigned)(nblk * cgs)), \
                       dim3(64 * WAVES), 0, st, s.data, d.data, (uint32_t)cpr, (uint32_t)cgs, s.ld, d.ld, tie)
    if (block == 32) MX_FQ_SPLIT(8, 4);
    else if (block == 64) MX_FQ_SPLIT(8, 8);
    else if (block == 128) MX_FQ_SPLIT(8, 16);
    else MX_FQ_SPLIT(4, 4);
#undef MX_FQ_SPLIT
  } else if (block != 32) {
    if (s.cols % 4 || s.rows % 32) return MX_ERR_UNSUPPORTED;
    const int64_t nrb = s.rows / 32, cgs = (s.cols + kColTileCols - 1) / kColTileCols, rbgs = (nrb + kColTileRbs - 1) / kColTileRbs;
    if (cgs * rbgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((fake_quant_cols_kblock_kernel<TARGET, ANCHOR, HW, DT>), dim3((unsigned)(cgs * rbgs)), dim3(256), 0, st, s.data,
                       d.data, s.cols, (uint32_t)cgs, s.ld, d.ld, nrb, tie, block);
  } else {
    if (s.cols % 4) return MX_ERR_UNSUPPORTED;
    int64_t qpr = s.cols / 4, nrb = s.rows / 32, nitems = qpr * nrb;
    if (qpr > 0xFFFFFFFFll) return MX_ERR_UNSUPPORTED;
    constexpr int kFqColsThreads = 128;  // two waves per workgroup stream this pattern best (78 % against 72 % with four)
    int64_t wgs = (nitems + kFqColsThreads - 1) / kFqColsThreads;
    if (wgs > 0x7FFFFFFF) return MX_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((fake_quant_cols_kernel<TARGET, ANCHOR, HW, DT, kFqColsThreads>), dim3((unsigned)wgs), dim3(kFqColsThreads), 0, st, s.data, d.data,
                       nitems, (uint32_t)qpr, s.ld, d.ld, tie);
  }
  return launch_status("a dense kernel");
}

// ---- runtime -> template dispatch
#define MX_FOR_EACH_ELEM(X)                                                                                   \
  X(MX_INT8) X(MX_INT7) X(MX_INT6) X(MX_INT5) X(MX_INT4) X(MX_INT3) X(MX_INT2) X(MX_FP8_E4M3) X(MX_FP7_E3M3) \
  X(MX_FP6_E3M2) X(MX_FP6_E2M3) X(MX_FP5_E2M2) X(MX_FP4_E2M1)

static inline bool use_hw(int elem_is_fp, int tie) { return elem_is_fp && (tie == MX_ROUND_DEFAULT || tie == MX_ROUND_HALF_EVEN); }

mx_status_t quantize_launch(int elem, int axis, int block, int tie, const DenseArg& src, void* codes, uint8_t* scales,
                            hipStream_t stream) {
#define X(ID)                                                                                              \
  if (elem == ID) {                                                                                        \
    constexpr bool CAN = Elem<ID>::hw != HW_NONE;                                                          \
    bool hw = CAN && use_hw(!Elem<ID>::is_int, tie);                                                       \
    if (src.dtype == MX_F32)                                                                               \
      return hw ? run_quantize<ID, CAN, MX_F32>(axis, block, tie, src, codes, scales, stream)                     \
                : run_quantize<ID, false, MX_F32>(axis, block, tie, src, codes, scales, stream);                  \
    return hw ? run_quantize<ID, CAN, MX_BF16>(axis, block, tie, src, codes, scales, stream)                      \
              : run_quantize<ID, false, MX_BF16>(axis, block, tie, src, codes, scales, stream);                   \
  }
  MX_FOR_EACH_ELEM(X)
#undef X
  return MX_ERR_FORMAT;
}

mx_status_t dequant_launch(int elem, int axis, int block, const void* codes, const uint8_t* scales, const DenseArg& dst,
                           hipStream_t stream) {
#define X(ID)                                                                               \
  if (elem == ID) {                                                                         \
    if (dst.dtype == MX_F32) return run_dequant<ID, MX_F32>(axis, block, codes, scales, dst, stream); \
    return run_dequant<ID, MX_BF16>(axis, block, codes, scales, dst, stream);                      \
  }
  MX_FOR_EACH_ELEM(X)
#undef X
  return MX_ERR_FORMAT;
}

template <int TARGET, int ANCHOR>
static mx_status_t fake_quant_pick(int axis, int block, int tie, const DenseArg& s, const DenseArg& d, hipStream_t stream) {
  constexpr bool CAN = Elem<TARGET>::hw != HW_NONE;  // the 8-bit FP anchor always has a hardware path
  bool hw = CAN && use_hw(!Elem<TARGET>::is_int, tie);
  if (s.dtype == MX_F32)
    return hw ? run_fake_quant<TARGET, ANCHOR, CAN, MX_F32>(axis, block, tie, s, d, stream)
              : run_fake_quant<TARGET, ANCHOR, false, MX_F32>(axis, block, tie, s, d, stream);
  return hw ? run_fake_quant<TARGET, ANCHOR, CAN, MX_BF16>(axis, block, tie, s, d, stream)
            : run_fake_quant<TARGET, ANCHOR, false, MX_BF16>(axis, block, tie, s, d, stream);
}

mx_status_t fake_quant_launch(int target, int anchor, int axis, int block, int tie, const DenseArg& src, const DenseArg& dst,
                              hipStream_t stream) {
#define X(ID)                                                                                             \
  if (target == ID) {                                                                                     \
    if (anchor < 0) return fake_quant_pick<ID, -1>(axis, block, tie, src, dst, stream);                          \
    if constexpr (Elem<ID>::is_int && Elem<ID>::bits < 8) {                                               \
      if (anchor == MX_INT8) return fake_quant_pick<ID, MX_INT8>(axis, block, tie, src, dst, stream);            \
    }                                                                                                     \
    if constexpr (!Elem<ID>::is_int && Elem<ID>::bits < 8) {                                              \
      if (anchor == MX_FP8_E4M3) return fake_quant_pick<ID, MX_FP8_E4M3>(axis, block, tie, src, dst, stream);    \
    }                                                                                                     \
    return MX_ERR_FORMAT;                                                                                 \
  }
  MX_FOR_EACH_ELEM(X)
#undef X
  return MX_ERR_FORMAT;
}

}  // namespace mx
