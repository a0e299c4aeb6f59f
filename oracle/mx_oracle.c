/*
 * mx_oracle.c -- CPU oracle for microscaling (MX) quantization, Slice-and-Scale,
 * dequantization and fake-quant.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, scalar
 * restatement of the method's definitions in double precision.  It shares no
 * code, header, table or constant with the HIP library; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it follows (paper sections):
 *   Sec. 3.3 notation: a block of k floats V_i becomes one shared scale X and k
 *     elements P_i, reconstruction V^_i = X * P_i.
 *   Eq. (1): shared_exp = floor(log2(max_i |V_i|)) - e_max(f),  X = 2^shared_exp.
 *   Eq. (2): P_i = quantize_f(V_i / X)  (rounding plus clamping).
 *   Sec. 3.3 "MXINT representation": P_i = clip_b(Round(V_i / X)).
 *   Eq. (4) SSMXINT: P_l = clip_bl(Round(P_h / 2^De)), X_l = X_h * 2^De, De = b_h - b_l.
 *   Eq. (6) SSMXFP : P_l = quantize_{eta_l,mu_l}(P_h / 2^De), X_l = X_h * 2^De,
 *                    De = e_max(eta_h) - e_max(eta_l).
 *   Eq. (7): W_A = Q_A(W_fp), W_t = Q_{A->t}(W_A); the model runs with W_t.
 *
 * Readings taken where the paper is silent (each listed in the design notes):
 *   - MXINT uses the integer view of the elements: e_max(b) = b - 2, so that
 *     De = b_h - b_l as the paper states below Eq. (3).
 *   - clip_b is symmetric: [-(2^(b-1)-1), 2^(b-1)-1].
 *   - Round for MXINT is round-half-away-from-zero (this is what "round using the
 *     most significant dropped bit" gives on magnitudes); quantize for MXFP is
 *     round-half-to-even on the target mantissa.  The tie argument can force
 *     either rule for either family.
 *   - MXFP quantize saturates the magnitude to the largest normal; it never
 *     emits a NaN code.  The sign of zero is kept.
 *   - All-zero block: scale byte 0, all codes 0.  A block that holds a NaN or an
 *     Inf: scale byte 255 (E8M0 NaN), all codes 0.
 *   - shared_exp is clamped to [-127, 127]; the stored byte is shared_exp + 127.
 *     Slice-and-Scale saturates byte + De at 254 and leaves 255 alone.
 *   - An E4M3 NaN code inside an anchor is sliced to +-max normal of a target
 *     that has no NaN, and stays NaN if the target is E4M3.
 *   - Sub-byte codes of one block are packed as a little-endian bit string:
 *     element i occupies bits [i*w, (i+1)*w).
 *   - Packed layout is block-contiguous: [outer][nblocks][bytes per block]; for
 *     axis 1 on a [rows, cols] matrix outer = rows, for axis 0 outer = cols.
 *
 * parity unpinned: the conventions above for the tie rule, the symmetric clip,
 * the all-zero block, the sign of zero and NaN/Inf handling have no value printed
 * in the paper to check against; everything else is pinned by tests/test_oracle_*.
 *
 * Element formats are passed as three ints (kind, a, b):
 *   kind 0: MXINT(b = a) signed integer elements, a in 2..8, b ignored.
 *   kind 1: MXFP(eta = a, mu = b): sign, eta exponent bits, mu mantissa bits.
 *           E4M3 reserves S.1111.111 for NaN (largest normal 448); every other
 *           (eta, mu) has neither Inf nor NaN.
 * tie: 0 = family default, 1 = half away from zero, 2 = half to even.
 * dtype: 0 = float32, 1 = bfloat16 (uint16 bit patterns).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define KIND_INT 0
#define KIND_FP 1

static int g_threads = 1;

void mxo_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int mxo_get_threads(void) {
#ifdef _OPENMP
    return g_threads;
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- formats */

int mxo_elem_bits(int kind, int a, int b) { return kind == KIND_INT ? a : 1 + a + b; }

static int fp_bias(int eta) { return (1 << (eta - 1)) - 1; }

static int fp_has_nan(int eta, int mu) { return eta == 4 && mu == 3; }

/* Exponent of the largest normal number of the element format (Sec. 3.3
 * notation).  MXINT(b): largest magnitude 2^(b-1)-1 lies in [2^(b-2), 2^(b-1)). */
int mxo_emax(int kind, int a, int b) {
    if (kind == KIND_INT) return a - 2;
    int top_field = (1 << a) - 1;          /* all-ones exponent field is a normal binade */
    (void)b;
    return top_field - fp_bias(a);
}

double mxo_max_normal(int kind, int a, int b) {
    if (kind == KIND_INT) return (double)((1 << (a - 1)) - 1);
    int top_m = (1 << b) - 1;
    if (fp_has_nan(a, b)) top_m -= 1;      /* the all-ones mantissa in the top binade is NaN */
    return ldexp(1.0 + (double)top_m / (double)(1 << b), mxo_emax(kind, a, b));
}

/* Value of one element code.  MXINT: two's complement in `a` bits.  MXFP:
 * (-1)^s 2^(E-bias) (1 + m/2^mu) for E > 0, (-1)^s 2^(1-bias) (m/2^mu) for E = 0. */
double mxo_decode(int kind, int a, int b, unsigned code) {
    if (kind == KIND_INT) {
        int bits = a;
        int v = (int)(code & ((1u << bits) - 1));
        if (v >= (1 << (bits - 1))) v -= (1 << bits);
        return (double)v;
    }
    int eta = a, mu = b;
    unsigned m = code & ((1u << mu) - 1);
    unsigned E = (code >> mu) & ((1u << eta) - 1);
    unsigned s = (code >> (mu + eta)) & 1u;
    double mag;
    if (fp_has_nan(eta, mu) && E == (1u << eta) - 1 && m == (1u << mu) - 1) return NAN;
    if (E == 0) mag = ldexp((double)m / (double)(1 << mu), 1 - fp_bias(eta));
    else mag = ldexp(1.0 + (double)m / (double)(1 << mu), (int)E - fp_bias(eta));
    return s ? -mag : mag;
}

static double round_tie(double q, int half_even) {
    /* q >= 0 and exactly representable; both functions are exact here */
    return half_even ? rint(q) /* default rounding mode: nearest even */ : round(q);
}

/* quantize_f(r): nearest element value, ties by `tie`, magnitude clamped to the
 * largest normal, returned as the element code (Eq. (2); Sec. 3.3 and 3.4). */
unsigned mxo_encode(int kind, int a, int b, double r, int tie) {
    if (kind == KIND_INT) {
        int bits = a;
        int half_even = (tie == 2);
        double lim = (double)((1 << (bits - 1)) - 1);
        double mag = round_tie(fabs(r), half_even);
        if (mag > lim) mag = lim;
        int v = (int)mag;
        if (r < 0) v = -v;
        return (unsigned)v & ((1u << bits) - 1);
    }
    int eta = a, mu = b;
    int half_even = (tie != 1);
    int bias = fp_bias(eta);
    unsigned s = signbit(r) ? 1u : 0u;
    double mag = fabs(r);
    double val = 0.0;
    if (mag > 0.0) {
        int e;
        (void)frexp(mag, &e);              /* mag = f * 2^e, f in [0.5, 1)  =>  floor(log2 mag) = e - 1 */
        e -= 1;
        if (e < 1 - bias) e = 1 - bias;    /* below the smallest normal the spacing stays that of the subnormals */
        double step = ldexp(1.0, e - mu);
        val = round_tie(mag / step, half_even) * step;
        double top = mxo_max_normal(kind, a, b);
        if (val > top) val = top;
    }
    unsigned E, m;
    if (val < ldexp(1.0, 1 - bias)) {
        E = 0;
        m = (unsigned)(val / ldexp(1.0, 1 - bias - mu));
    } else {
        int e;
        (void)frexp(val, &e);
        e -= 1;
        E = (unsigned)(e + bias);
        m = (unsigned)((val / ldexp(1.0, e) - 1.0) * (double)(1 << mu));
    }
    return (s << (eta + mu)) | (E << mu) | m;
}

/* ----------------------------------------------------------------- scales */

/* Eq. (1) for one block, returned as the stored E8M0 byte = shared_exp + 127. */
int mxo_scale_byte(double amax, int kind, int a, int b) {
    if (isnan(amax) || isinf(amax)) return 255;
    if (amax == 0.0) return 0;
    int e;
    (void)frexp(amax, &e);
    int shared_exp = (e - 1) - mxo_emax(kind, a, b);
    if (shared_exp < -127) shared_exp = -127;
    if (shared_exp > 127) shared_exp = 127;
    return shared_exp + 127;
}

double mxo_scale_value(int byte) { return byte == 255 ? NAN : ldexp(1.0, byte - 127); }

/* De of Eq. (4) / Eq. (6). */
int mxo_delta_e(int kind, int ah, int bh, int al, int bl) {
    return mxo_emax(kind, ah, bh) - mxo_emax(kind, al, bl);
}

/* ------------------------------------------------------------ bit packing */

static long block_bytes(int k, int bits) { return ((long)k * bits + 7) / 8; }

long mxo_block_bytes(int k, int bits) { return block_bytes(k, bits); }

/* codes: one element code per byte; out: bit string, element i at bits [i*w,(i+1)*w) */
void mxo_pack_block(const uint8_t* codes, int k, int bits, uint8_t* out) {
    memset(out, 0, (size_t)block_bytes(k, bits));
    for (int i = 0; i < k; ++i)
        for (int j = 0; j < bits; ++j)
            if ((codes[i] >> j) & 1u) {
                long pos = (long)i * bits + j;
                out[pos >> 3] |= (uint8_t)(1u << (pos & 7));
            }
}

void mxo_unpack_block(const uint8_t* in, int k, int bits, uint8_t* codes) {
    for (int i = 0; i < k; ++i) {
        unsigned c = 0;
        for (int j = 0; j < bits; ++j) {
            long pos = (long)i * bits + j;
            if ((in[pos >> 3] >> (pos & 7)) & 1u) c |= 1u << j;
        }
        codes[i] = (uint8_t)c;
    }
}

/* ------------------------------------------------------------ block steps */

/* Eq. (1) + Eq. (2) on one block of k doubles. codes: one per byte. */
void mxo_quantize_block(const double* V, int k, int kind, int a, int b, int tie,
                        uint8_t* codes, uint8_t* byte_out) {
    double amax = 0.0;
    int bad = 0;
    for (int i = 0; i < k; ++i) {
        if (isnan(V[i]) || isinf(V[i])) bad = 1;
        else if (fabs(V[i]) > amax) amax = fabs(V[i]);
    }
    int byte = bad ? 255 : mxo_scale_byte(amax, kind, a, b);
    *byte_out = (uint8_t)byte;
    if (byte == 255) { memset(codes, 0, (size_t)k); return; }
    int shared_exp = byte - 127;
    for (int i = 0; i < k; ++i) {
        double r = ldexp(V[i], -shared_exp);   /* V_i / X, exact */
        codes[i] = (uint8_t)mxo_encode(kind, a, b, r, tie);
    }
}

/* Eq. (4) / Eq. (6) element step for one anchor code. */
unsigned mxo_slice_code(int kind, int ah, int bh, int al, int bl, int tie, unsigned code_h) {
    int de = mxo_delta_e(kind, ah, bh, al, bl);
    double p = mxo_decode(kind, ah, bh, code_h);
    if (isnan(p)) {                            /* E4M3 NaN element inside an anchor */
        unsigned s = (code_h >> 7) & 1u;
        if (kind == KIND_FP && fp_has_nan(al, bl)) return (s << 7) | 0x7Fu;
        p = s ? -mxo_max_normal(kind, ah, bh) : mxo_max_normal(kind, ah, bh);
    }
    return mxo_encode(kind, al, bl, ldexp(p, -de), tie);
}

/* Eq. (4) / Eq. (6) scale step. */
int mxo_slice_byte(int kind, int ah, int bh, int al, int bl, int byte_h) {
    if (byte_h == 255) return 255;
    int v = byte_h + mxo_delta_e(kind, ah, bh, al, bl);
    return v > 254 ? 254 : v;
}

/* V^_i = X * P_i (Sec. 3.3 notation), as a double (NaN when the scale byte is 255). */
double mxo_dequant_value(int kind, int a, int b, unsigned code, int byte) {
    if (byte == 255) return NAN;
    double p = mxo_decode(kind, a, b, code);
    return ldexp(p, byte - 127);
}

/* ----------------------------------------------------- dense element types */

static double bf16_bits_to_double(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* nearest bfloat16 (8 significant bits, fp32 exponent range), ties to even */
static uint16_t double_to_bf16_bits(double v) {
    if (isnan(v)) return 0x7FC0;
    uint16_t s = signbit(v) ? 0x8000 : 0;
    double mag = fabs(v);
    if (mag == 0.0) return s;
    if (isinf(mag)) return (uint16_t)(s | 0x7F80);
    int e;
    (void)frexp(mag, &e);
    e -= 1;
    if (e < -126) e = -126;
    double step = ldexp(1.0, e - 7);
    double q = rint(mag / step) * step;
    if (q >= ldexp(1.0, 128)) return (uint16_t)(s | 0x7F80);
    float f = (float)q;                        /* exact: q has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(s | (u >> 16));
}

static double load_dense(const void* p, int dtype, long idx) {
    if (dtype == 0) return (double)((const float*)p)[idx];
    return bf16_bits_to_double(((const uint16_t*)p)[idx]);
}

static void store_dense(void* p, int dtype, long idx, double v) {
    if (dtype == 0) ((float*)p)[idx] = (float)v;   /* nearest fp32, overflow -> Inf */
    else ((uint16_t*)p)[idx] = double_to_bf16_bits(v);
}

uint16_t mxo_double_to_bf16(double v) { return double_to_bf16_bits(v); }
double mxo_bf16_to_double(uint16_t h) { return bf16_bits_to_double(h); }

/* ------------------------------------------------------------ tensor steps */

/* Address of element i of block (o, j): axis 1 -> row o, col j*k+i; axis 0 -> row j*k+i, col o. */
static long dense_index(long o, long j, int i, int k, int axis, long ld) {
    if (axis == 1) return o * ld + j * k + i;
    return (j * k + i) * ld + o;
}

static int check_shape(long rows, long cols, long ld, int axis, int k, long* outer, long* nblk) {
    if (rows < 0 || cols < 0 || k < 1 || k > 1024 || ld < cols) return -1;
    if (axis == 1) { if (cols % k) return -1; *outer = rows; *nblk = cols / k; }
    else if (axis == 0) { if (rows % k) return -1; *outer = cols; *nblk = rows / k; }
    else return -1;
    return 0;
}

/* Q_f over a [rows, cols] matrix (leading dimension ld, in elements). */
int mxo_quantize(const void* src, int dtype, long rows, long cols, long ld, int axis, int k,
                 int kind, int a, int b, int tie, uint8_t* codes, uint8_t* scales) {
    long outer, nblk;
    if (check_shape(rows, cols, ld, axis, k, &outer, &nblk)) return -1;
    int bits = mxo_elem_bits(kind, a, b);
    long bb = block_bytes(k, bits);
    long total = outer * nblk;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (long t = 0; t < total; ++t) {
        long o = t / nblk, j = t % nblk;
        double V[1024];
        uint8_t c[1024];
        for (int i = 0; i < k; ++i) V[i] = load_dense(src, dtype, dense_index(o, j, i, k, axis, ld));
        mxo_quantize_block(V, k, kind, a, b, tie, c, &scales[t]);
        mxo_pack_block(c, k, bits, codes + t * bb);
    }
    return 0;
}

/* Q_{A->t} over a flat run of blocks (the packed layout makes the axis irrelevant). */
int mxo_slice_and_scale(int kind, int ah, int bh, int al, int bl, int tie, int k, long nblocks,
                        const uint8_t* codes_h, const uint8_t* scales_h,
                        uint8_t* codes_l, uint8_t* scales_l) {
    if (nblocks < 0 || k < 1 || k > 1024) return -1;
    int bits_h = mxo_elem_bits(kind, ah, bh), bits_l = mxo_elem_bits(kind, al, bl);
    long bbh = block_bytes(k, bits_h), bbl = block_bytes(k, bits_l);
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (long t = 0; t < nblocks; ++t) {
        uint8_t ch[1024], cl[1024];
        mxo_unpack_block(codes_h + t * bbh, k, bits_h, ch);
        for (int i = 0; i < k; ++i) cl[i] = (uint8_t)mxo_slice_code(kind, ah, bh, al, bl, tie, ch[i]);
        mxo_pack_block(cl, k, bits_l, codes_l + t * bbl);
        scales_l[t] = (uint8_t)mxo_slice_byte(kind, ah, bh, al, bl, scales_h[t]);
    }
    return 0;
}

/* V^ = X * P written to a dense [rows, cols] matrix. */
int mxo_dequant(int kind, int a, int b, int k, const uint8_t* codes, const uint8_t* scales,
                long rows, long cols, long ld, int axis, int dtype, void* dst) {
    long outer, nblk;
    if (check_shape(rows, cols, ld, axis, k, &outer, &nblk)) return -1;
    int bits = mxo_elem_bits(kind, a, b);
    long bb = block_bytes(k, bits);
    long total = outer * nblk;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (long t = 0; t < total; ++t) {
        long o = t / nblk, j = t % nblk;
        uint8_t c[1024];
        mxo_unpack_block(codes + t * bb, k, bits, c);
        for (int i = 0; i < k; ++i)
            store_dense(dst, dtype, dense_index(o, j, i, k, axis, ld),
                        mxo_dequant_value(kind, a, b, c[i], scales[t]));
    }
    return 0;
}

/* Fake-quant: dst = DQ(Q_t(src)) when has_anchor == 0 (Sec. 3.2), else
 * dst = DQ(Q_{A->t}(Q_A(src))) (Eq. (7)).  The target is (kind, al, bl), the
 * anchor (kind, ah, bh). */
int mxo_fake_quant(int kind, int al, int bl, int has_anchor, int ah, int bh, int tie, int k,
                   const void* src, int dtype, long rows, long cols, long ld, int axis,
                   int dst_dtype, void* dst, long dst_ld) {
    long outer, nblk;
    if (check_shape(rows, cols, ld, axis, k, &outer, &nblk)) return -1;
    if (dst_ld < cols) return -1;
    long total = outer * nblk;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (long t = 0; t < total; ++t) {
        long o = t / nblk, j = t % nblk;
        double V[1024];
        uint8_t c[1024], c2[1024], byte;
        for (int i = 0; i < k; ++i) V[i] = load_dense(src, dtype, dense_index(o, j, i, k, axis, ld));
        if (!has_anchor) {
            mxo_quantize_block(V, k, kind, al, bl, tie, c, &byte);
        } else {
            uint8_t byte_h;
            mxo_quantize_block(V, k, kind, ah, bh, tie, c2, &byte_h);
            for (int i = 0; i < k; ++i) c[i] = (uint8_t)mxo_slice_code(kind, ah, bh, al, bl, tie, c2[i]);
            byte = (uint8_t)mxo_slice_byte(kind, ah, bh, al, bl, byte_h);
        }
        for (int i = 0; i < k; ++i)
            store_dense(dst, dst_dtype, dense_index(o, j, i, k, axis, dst_ld),
                        mxo_dequant_value(kind, al, bl, c[i], byte));
    }
    return 0;
}
