// fcv2_bits.h -- integer building blocks of the codec kernels: bf16 bit handling, order keys, and the
// shift/mask sequences that move code fields between "one code per byte" registers and the packed bit planes
// (Section 3.2 of arxiv 2508.03760: a b-bit code is split into 4/2/1-bit planes stored separately).
//
// Everything here is plain 32-bit integer arithmetic, usable from host and device, so the sequences can be
// unit-tested on the CPU.  A lane of the kernels always works on 8 consecutive elements:
//   c0 = codes of elements 0..3, one per byte (element 0 in bits 0..7), c1 = elements 4..7.
#pragma once
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define FCV2_HD __host__ __device__ __forceinline__
#else
#define FCV2_HD inline
#endif

// Tables and the functions that index them: device-only inside the HIP translation unit, plain host code in
// the CPU test build.
#if defined(__HIPCC__)
#define FCV2_TABLE static __device__ const
#define FCV2_D __device__ __forceinline__
#else
#define FCV2_TABLE static const
#define FCV2_D inline
#endif

// Keeps the compiler from merging a chain of shift-or steps into one 32-bit multiply (quarter rate on CDNA).
#if defined(__HIP_DEVICE_COMPILE__)
#define FCV2_KEEP(v) asm volatile("" : "+v"(v))
#else
#define FCV2_KEEP(v) (void)(v)
#endif

namespace fcv2 {

// ---- single instructions whose form matters --------------------------------------------------------------------------
// Measured on the MI355X (8 waves per SIMD, independent chains): a wave-wide VALU instruction issues in about 2.4
// cycles when it is a two-operand instruction of a simple class -- and, or, xor, right shift, integer add, fp32
// add / subtract / multiply, move -- whose operands are vector registers, a literal or an inline constant; in about 3
// cycles for an fp32 FMA and for v_bitop3 on three vector registers; and in about 4.2 cycles otherwise: anything that
// reads a SCALAR register, left shifts, the three-operand integer forms, integer min/max/med3, conversions, packed
// 16-bit, DPP, SDWA, permutes, dot products (reciprocal: 8.3).  The compiler likes to park a constant that is used
// more than once in a scalar register, which turns the cheapest class into the dearest; the helpers below pin the
// cheap form.  On the host they are plain C.
#if defined(__HIP_DEVICE_COMPILE__)
template <uint32_t C> FCV2_D uint32_t and_lit(uint32_t x) {  // x & C as v_and_b32 with the literal in the instruction
    uint32_t r;
    asm("v_and_b32 %0, %1, %2" : "=v"(r) : "n"((int32_t)C), "v"(x));
    return r;
}
template <uint32_t C> FCV2_D uint32_t xor_lit(uint32_t x) {
    uint32_t r;
    asm("v_xor_b32 %0, %1, %2" : "=v"(r) : "n"((int32_t)C), "v"(x));
    return r;
}
// A constant held in a vector register the compiler cannot see through (so it cannot move it to a scalar one).
template <uint32_t C> FCV2_D uint32_t vreg_const() {
    uint32_t r;
    asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "n"((int32_t)C));
    return r;
}
// (m & a) | (~m & b) in one v_bitop3 on three vector registers.
FCV2_D uint32_t bit_select(uint32_t m, uint32_t a, uint32_t b) { return __builtin_amdgcn_bitop3_b32(a, b, m, 0xE4); }
// (a | b) & m likewise.
FCV2_D uint32_t or_and(uint32_t a, uint32_t b, uint32_t m) { return __builtin_amdgcn_bitop3_b32(a, b, m, 0xA8); }
// sum of byte products: a.b0 * w.b0 + ... + a.b3 * w.b3 + c
FCV2_D uint32_t dot4_u8(uint32_t a, uint32_t w, uint32_t c) { return __builtin_amdgcn_udot4(a, w, c, false); }
FCV2_D uint32_t rotr32(uint32_t x, int r) { return __builtin_amdgcn_alignbit(x, x, r); }
#else  // the host pass of the HIP compiler, and the CPU test build
template <uint32_t C> FCV2_HD uint32_t and_lit(uint32_t x) { return x & C; }
template <uint32_t C> FCV2_HD uint32_t xor_lit(uint32_t x) { return x ^ C; }
template <uint32_t C> FCV2_HD uint32_t vreg_const() { return C; }
FCV2_HD uint32_t bit_select(uint32_t m, uint32_t a, uint32_t b) { return (m & a) | (~m & b); }
FCV2_HD uint32_t or_and(uint32_t a, uint32_t b, uint32_t m) { return (a | b) & m; }
FCV2_HD uint32_t dot4_u8(uint32_t a, uint32_t w, uint32_t c) {
    for (int i = 0; i < 4; ++i) c += ((a >> (8 * i)) & 0xFFu) * ((w >> (8 * i)) & 0xFFu);
    return c;
}
FCV2_HD uint32_t rotr32(uint32_t x, int r) { return (x >> r) | (x << ((32 - r) & 31)); }
#endif

// ---- plane structure of a b-bit code: widest plane first = most significant bits ---------------------------
template <int BITS> struct Planes;
template <> struct Planes<2> { static constexpr int w8 = 0, w4 = 0, w2 = 1, w1 = 0, sh4 = 0, sh2 = 0, sh1 = 0; };
template <> struct Planes<3> { static constexpr int w8 = 0, w4 = 0, w2 = 1, w1 = 1, sh4 = 0, sh2 = 1, sh1 = 0; };
template <> struct Planes<4> { static constexpr int w8 = 0, w4 = 1, w2 = 0, w1 = 0, sh4 = 0, sh2 = 0, sh1 = 0; };
template <> struct Planes<5> { static constexpr int w8 = 0, w4 = 1, w2 = 0, w1 = 1, sh4 = 1, sh2 = 0, sh1 = 0; };
template <> struct Planes<6> { static constexpr int w8 = 0, w4 = 1, w2 = 1, w1 = 0, sh4 = 2, sh2 = 0, sh1 = 0; };
template <> struct Planes<7> { static constexpr int w8 = 0, w4 = 1, w2 = 1, w1 = 1, sh4 = 3, sh2 = 1, sh1 = 0; };
template <> struct Planes<8> { static constexpr int w8 = 1, w4 = 0, w2 = 0, w1 = 0, sh4 = 0, sh2 = 0, sh1 = 0; };

// ---- bf16 ---------------------------------------------------------------------------------------------------
// Total order on bf16 bit patterns that equals numeric order on finite values, with -0 below +0.
FCV2_HD uint32_t key_of_bf16(uint32_t u) { return (u & 0x8000u) ? (~u & 0xFFFFu) : (u | 0x8000u); }
FCV2_HD uint32_t bf16_of_key(uint32_t k) { return (k & 0x8000u) ? (k ^ 0x8000u) : (~k & 0xFFFFu); }

// fp32 bits -> bf16 bits, round to nearest even; NaN stays a quiet NaN.
FCV2_HD uint32_t bf16_rne_bits(uint32_t u) {
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Smallest bf16-representable fp32 bit pattern that is >= the (positive, finite) input.
FCV2_HD uint32_t bf16_round_up_bits(uint32_t u) { return (u + 0xFFFFu) & 0xFFFF0000u; }

// d / QMAX with IEEE rounding for d >= 0, without the long division sequence: multiply by the rounded
// reciprocal, then one exact-residual correction (Markstein).  Checked against IEEE division for every fp32
// significand and every QMAX = 2^b - 1 by the host tests; +inf and NaN are passed through.
template <int QMAX> FCV2_HD float div_by_qmax(float d) {
    constexpr float y = 1.0f / (float)QMAX;
    const float q0 = d * y;
    const float r = fmaf(-(float)QMAX, q0, d);
    const float q1 = fmaf(r, y, q0);
    return (d < INFINITY) ? q1 : d;
}

// ---- integer metadata (Section 3.3, Eq. 1: scale_int = round(log2(scale) * 10), one signed byte) -------------
// kPow10th[j + 1] = 2^(j/10) rounded to fp32 for j = -1..10.  kThr10th[j] = 2^((j - 1/2)/10) rounded UP to fp32 for
// j = 0..10: a scale s has round(log2(s) * 10) >= 10e + j exactly when s >= 2^e * kThr10th[j] (the true thresholds
// are irrational, so rounding them up to the next fp32 changes no decision).
#define FCV2_POW10TH_VALUES                                                                                                    \
    {0x1.ddb680p-1f, 0x1.000000p+0f, 0x1.125fbep+0f, 0x1.261118p+0f, 0x1.3b2c48p+0f, 0x1.51cb46p+0f,                               \
     0x1.6a09e6p+0f, 0x1.840600p+0f, 0x1.9fdf8cp+0f, 0x1.bdb8cep+0f, 0x1.ddb680p+0f, 0x1.000000p+1f}
#define FCV2_THR10TH_VALUES                                                                                                    \
    {0x1.ee8f36p-1f, 0x1.090720p+0f, 0x1.1c0cc0p+0f, 0x1.306fe2p+0f, 0x1.46499cp+0f, 0x1.5db4d2p+0f,                               \
     0x1.76ce52p+0f, 0x1.91b502p+0f, 0x1.ae89fap+0f, 0x1.cd70b4p+0f, 0x1.ee8f36p+0f}
FCV2_TABLE float kPow10th[12] = FCV2_POW10TH_VALUES;
FCV2_TABLE float kThr10th[11] = FCV2_THR10TH_VALUES;

// k = 10e + j with 0 <= j <= 9, for -128 <= k <= 127.
FCV2_D void split_tenths(int k, int& e, int& j) {
    const uint32_t u = (uint32_t)(k + 130);
    const uint32_t q = (u * 205u) >> 11;  // u / 10 for u < 1029
    e = (int)q - 13;
    j = (int)(u - 10u * q);
}

// The scale a receiver reconstructs from the byte: 2^(k/10) as an fp32 value (the table entry scaled by an exact
// power of two).
FCV2_D float scale_of_int(int k) {
    int e, j;
    split_tenths(k, e, j);
    return ldexpf(kPow10th[j + 1], e);
}

// round(log2(s) * 10) to within 1 from the bit pattern alone: exponent + significand fraction is a piecewise-linear
// log2 that is low by at most 0.0861; centring that error leaves |10 * error| < 0.44, so the rounded estimate is
// at most one off.
FCV2_D int scale_int_estimate(float s) {
    uint32_t bits;
    __builtin_memcpy(&bits, &s, 4);
    const float t = (float)((int32_t)bits - 0x3F800000) * (10.0f / 8388608.0f) + 0.43f;
    return (int)rintf(fminf(fmaxf(t, -128.0f), 127.0f));
}

struct ScaleInt {
    int k;    // Eq. 1, clamped to a signed byte
    float s;  // 2^(k/10)
};

// Eq. 1 without a logarithm: the estimate is corrected by comparing s with the two thresholds around it.
// Zero, negative and NaN inputs give the lowest code.
FCV2_D ScaleInt scale_int_of(float s) {
    int k0 = (s > 0.0f) ? scale_int_estimate(s) : -128;
    int e, j;
    split_tenths(k0, e, j);
    const float below = ldexpf(kThr10th[j], e), above = ldexpf(kThr10th[j + 1], e);
    int d = 0;
    if (s >= above) d = 1;
    if (s < below) d = -1;
    if (k0 + d > 127 || k0 + d < -128) d = 0;
    ScaleInt r;
    r.k = k0 + d;
    r.s = ldexpf(kPow10th[j + 1 + d], e);
    return r;
}

// The same two functions from per-code tables (the kernels keep them in LDS): pow_tab[k + 129] = 2^(k/10) for
// k = -128..127 (entries 0 and 257 are never selected, they only keep the neighbour reads in bounds),
// thr_tab[k + 128] = smallest fp32 whose code is >= k, for k = -128..128.  Entry t of each:
FCV2_D float scale_table_pow(int t) { return (t >= 1 && t <= 256) ? scale_of_int(t - 129) : 0.0f; }
FCV2_D float scale_table_thr(int t) {
    int e, j;
    split_tenths(t - 128, e, j);  // the split also holds for k = 128
    return ldexpf(kThr10th[j], e);
}
constexpr int kScaleTablePow = 258, kScaleTableThr = 257;

// Both tables written out at compile time, the power table first: what a kernel copies into LDS.  An entry is one of the
// twelve (eleven) values above times an exact power of two between 2^-13 and 2^13, so the products are the values that
// scale_table_pow and scale_table_thr compute (the host tests compare all of them).
struct ScaleTables {
    float v[kScaleTablePow + kScaleTableThr];
};
constexpr float exact_pow2(int e) {
    float r = 1.0f;
    for (; e > 0; --e) r *= 2.0f;
    for (; e < 0; ++e) r *= 0.5f;
    return r;
}
constexpr ScaleTables make_scale_tables() {
    constexpr float pow10th[12] = FCV2_POW10TH_VALUES;
    constexpr float thr10th[11] = FCV2_THR10TH_VALUES;
    ScaleTables T{};
    for (int t = 0; t < kScaleTablePow + kScaleTableThr; ++t) {
        const bool is_pow = t < kScaleTablePow;
        const int k = is_pow ? t - 129 : t - kScaleTablePow - 128;  // the code the entry belongs to
        const int u = k + 130, q = (u * 205) >> 11, e = q - 13, j = u - 10 * q;  // split_tenths
        T.v[t] = is_pow ? ((t >= 1 && t <= 256) ? pow10th[j + 1] * exact_pow2(e) : 0.0f) : thr10th[j] * exact_pow2(e);
    }
    return T;
}
FCV2_TABLE ScaleTables kScaleTablesInit = make_scale_tables();

FCV2_D ScaleInt scale_int_from_tables(float s, const float* pow_tab, const float* thr_tab) {
    const int k0 = (s > 0.0f) ? scale_int_estimate(s) : -128;
    const float below = thr_tab[k0 + 128], above = thr_tab[k0 + 129];
    int d = 0;
    if (s >= above) d = 1;
    if (s < below) d = -1;
    if (k0 + d > 127 || k0 + d < -128) d = 0;
    ScaleInt r;
    r.k = k0 + d;
    r.s = pow_tab[k0 + 129 + d];
    return r;
}

// ---- launch plan of the row-staged dispatch kernel (host) ---------------------------------------------------------
// A block takes `rows` consecutive tokens of `lpr` lanes each (a lane = 32 elements) and has `threads` = their lanes
// rounded up to whole waves, at most 8 waves.  Its LDS holds a transpose scratch per wave, the packed records, the
// destination rows, the E expert starts (+ 8 words for the block scan) and, for integer metadata, the scale tables;
// 64 KiB at most.  Among the row counts 1..64 that fit, the one with the smallest share of idle lanes wins (the first
// such).  rows = 0: the shape does not fit the kernel.
constexpr uint32_t kWaveScratchBytes = 4096, kRowsPlanThreadsMax = 512;
struct RowsPlan {
    uint32_t rows, threads;
    size_t lds_bytes;
};
static inline RowsPlan rows_plan(uint32_t lpr, uint32_t K, uint32_t row_bytes, bool int_meta, uint32_t E) {
    // Candidates: R rows per block, as many whole waves as they need.  First choice: the count with the fewest idle lanes
    // (the smallest such count).  If that block is larger than four waves and a smaller count fills at least four waves
    // with at most an eighth of their lanes idle, the smallest such count is taken instead: smaller blocks finish their
    // load - quantize - copy sequence sooner (measured on 7168-element rows: one row in four waves, 32 lanes idle,
    // 62.3 us for the call, against two rows in seven full waves, 64.4 us).
    RowsPlan best = {0, 0, 0}, small = {0, 0, 0};
    uint32_t best_idle = ~0u;
    for (uint32_t R = 1; R <= 64 && R * lpr <= kRowsPlanThreadsMax; ++R) {
        const uint32_t waves = (R * lpr + 63) / 64;
        const size_t lds = (size_t)waves * kWaveScratchBytes + (size_t)R * row_bytes + (size_t)R * K * 4 + ((size_t)E + 8) * 4 +
                           (int_meta ? (size_t)(kScaleTablePow + kScaleTableThr) * 4 : 0);
        if (lds > 64 * 1024) break;
        const uint32_t idle = (waves * 64 - R * lpr) * 1024 / (waves * 64);  // idle lanes, in 1/1024 of the block
        if (idle < best_idle) {
            best_idle = idle;
            best = {R, waves * 64, lds};
        }
        if (small.rows == 0 && waves >= 4 && idle <= 128) small = {R, waves * 64, lds};
    }
    if (best.threads > 4 * 64 && small.rows != 0 && small.rows < best.rows) return small;
    return best;
}

// ---- codes (one per byte) -> planes ---------------------------------------------------------------------------
// Field (code >> SH) & (2^W - 1) of each byte, moved to the top W bits of that byte.
template <int W, int SH, int BITS> FCV2_HD uint32_t top_align(uint32_t c) {
    constexpr int lsh = 8 - W - SH;
    constexpr uint32_t m = (((0xFFu << (8 - W)) & 0xFFu) * 0x01010101u);
    uint32_t f = lsh > 0 ? (c << (lsh > 0 ? lsh : 0)) : c;
    // when the field reaches up to the top bit of the code nothing can spill into the next byte
    return (SH + W == BITS && SH == 0) ? f : (f & m);
}

// 8 nibbles: bits 4i..4i+3 = field of element i.
template <int SH, int BITS> FCV2_HD uint32_t pack_plane4(uint32_t c0, uint32_t c1) {
    uint32_t f0 = top_align<4, SH, BITS>(c0), f1 = top_align<4, SH, BITS>(c1);
    uint32_t a0 = (f0 << 4) | f0;  // bytes 1 and 3 hold (e0 | e1 << 4) and (e2 | e3 << 4)
    uint32_t a1 = (f1 << 4) | f1;
    return ((a0 >> 8) & 0xFFu) | ((a0 >> 16) & 0xFF00u) | ((a1 << 8) & 0xFF0000u) | (a1 & 0xFF000000u);
}

// 8 two-bit fields: bits 2i..2i+1 = field of element i (16 bits, nothing above them).  The four fields of a register
// are gathered by one byte dot product with the weights 1, 4, 16, 64 (the masked bytes are field << SH, so the sum is
// the packed byte << SH).
template <int SH, int BITS> FCV2_HD uint32_t pack_plane2(uint32_t c0, uint32_t c1) {
    constexpr uint32_t W = 0x40100401u;
    const uint32_t m0 = (BITS == 2) ? c0 : and_lit<(0x03030303u << SH)>(c0);
    const uint32_t m1 = (BITS == 2) ? c1 : and_lit<(0x03030303u << SH)>(c1);
    const uint32_t d0 = dot4_u8(m0, W, 0u), d1 = dot4_u8(m1, W, 0u);
    return ((d1 << 8) | d0) >> SH;
}

// 8 one-bit fields: bit i = field of element i (8 bits, nothing above them): two byte dot products with the weights 1, 2, 4, 8 and
// 16, 32, 64, 128, the second adding to the first.  The 1-bit plane always holds bit 0 of the code.
template <int SH, int BITS> FCV2_HD uint32_t pack_plane1(uint32_t c0, uint32_t c1) {
    static_assert(SH == 0, "the 1-bit plane is the least significant bit of the code");
    const uint32_t d = dot4_u8(and_lit<0x01010101u>(c0), 0x08040201u, 0u);
    return dot4_u8(and_lit<0x01010101u>(c1), 0x80402010u, d);
}

// ---- planes -> codes --------------------------------------------------------------------------------------------
// 8 one-bit fields (bit i) -> 8 nibbles (bit 4i).
FCV2_HD uint32_t spread1to4(uint32_t x) {
    x = (x | (x << 12)) & 0x000F000Fu;
    x = (x | (x << 6)) & 0x03030303u;
    x = (x | (x << 3)) & 0x11111111u;
    return x;
}
// 8 two-bit fields (bits 2i) -> 8 nibbles (bits 4i).
FCV2_HD uint32_t spread2to4(uint32_t x) {
    x = (x | (x << 8)) & 0x00FF00FFu;
    x = (x | (x << 4)) & 0x0F0F0F0Fu;
    x = (x | (x << 2)) & 0x33333333u;
    return x;
}

// Codes of the 8 elements as two "even/odd" registers: ev = elements 0,2,4,6 one per byte, od = 1,3,5,7.
// p4 / p2 / p1 are the lane's 32 / 16 / 8 bits of the planes; for BITS == 8 use the plane bytes directly.
template <int BITS> FCV2_HD void codes_even_odd(uint32_t p4, uint32_t p2, uint32_t p1, uint32_t& ev, uint32_t& od) {
    using P = Planes<BITS>;
    constexpr uint32_t M = 0x0F0F0F0Fu;
    uint32_t low = 0;  // nibble word of the planes below the 4-bit plane
    if (P::w2) low = spread2to4(p2) << P::sh2;
    if (P::w1) low |= spread1to4(p1);
    if (P::w4) {
        ev = ((p4 & M) << P::sh4) | (low & M);
        od = (((p4 >> 4) & M) << P::sh4) | ((low >> 4) & M);
    } else {
        ev = low & M;
        od = (low >> 4) & M;
    }
    FCV2_KEEP(ev);  // consumers convert byte k directly (v_cvt_f32_ubyte<k>); do not re-derive from the nibbles
    FCV2_KEEP(od);
}

// Codes of 8 elements as four "pair" registers: Q[k] holds element k in bits 0..15 and element k+4 in bits
// 16..31, each zero-extended.  Read as an fp16 denormal, a 16-bit integer q is exactly q * 2^-24, which lets a
// mixed-precision FMA consume the code without a separate integer-to-float conversion.
// p8lo/p8hi: the 8 plane-8 bytes; p4 / p2 / p1: the 32 / 16 / 8 bits of the other planes.
template <int BITS> FCV2_HD void codes_pairs(uint32_t p8lo, uint32_t p8hi, uint32_t p4, uint32_t p2, uint32_t p1, uint32_t (&Q)[4]) {
    using P = Planes<BITS>;
    if (P::w8) {
#if defined(__HIP_DEVICE_COMPILE__)
        Q[0] = __builtin_amdgcn_perm(p8hi, p8lo, 0x0C040C00u);
        Q[1] = __builtin_amdgcn_perm(p8hi, p8lo, 0x0C050C01u);
        Q[2] = __builtin_amdgcn_perm(p8hi, p8lo, 0x0C060C02u);
        Q[3] = __builtin_amdgcn_perm(p8hi, p8lo, 0x0C070C03u);
#else
        for (int k = 0; k < 4; ++k) Q[k] = ((p8lo >> (8 * k)) & 0xFFu) | (((p8hi >> (8 * k)) & 0xFFu) << 16);
#endif
        return;
    }
    // element k of the low half and element k+4 of the high half sit at the same offset inside their halves
    const uint32_t A2 = P::w2 ? ((p2 << 8) | p2) : 0u;   // bits 0..7: fields 0..3, bits 16..23: fields 4..7
    const uint32_t A1 = P::w1 ? ((p1 << 12) | p1) : 0u;  // bits 0..3: fields 0..3, bits 16..19: fields 4..7
#define FCV2_SHIFTED(x, amount) ((amount) >= 0 ? ((x) >> ((amount) >= 0 ? (amount) : 0)) : ((x) << ((amount) < 0 ? -(amount) : 0)))
    for (int k = 0; k < 4; ++k) {
        uint32_t q = 0;
        if (P::w4) q |= FCV2_SHIFTED(p4, 4 * k - P::sh4) & (0x000F000Fu << P::sh4);
        if (P::w2) q |= FCV2_SHIFTED(A2, 2 * k - P::sh2) & (0x00030003u << P::sh2);
        if (P::w1) q |= FCV2_SHIFTED(A1, k - P::sh1) & (0x00010001u << P::sh1);
        Q[k] = q;
    }
#undef FCV2_SHIFTED
}

// ---- 16 elements of a lane -> 8 registers of (element | element) 16-bit halves, for 2, 3 and 4 bits --------------
// As above, but the fields are only masked, never moved to bit 0: each half ends up holding code << pos with
// zeros around it, and the consumer folds 2^-pos into the scale it multiplies the half with (a half read as an
// fp16 denormal is an exact integer multiple of 2^-24 at any position below bit 10).  PairMap says which element
// sits where.  p2 = 32 bits (elements 0..15), p1 = 16 bits, p4a/p4b = elements 0..7 / 8..15.
template <int BITS> struct PairMap;
template <> struct PairMap<2> {  // 2-bit fields at offset 2e: direct for e = 0..4 (with e + 8), rotated by 10 for 5..7
    static constexpr int n_pos = 5;
    static constexpr int lo(int k) { return k; }
    static constexpr int hi(int k) { return k + 8; }
    static constexpr int pos(int k) { return k < 5 ? 2 * k : 2 * (k - 5); }
    static constexpr int k_of(int e) { return e & 7; }       // the register that holds element e ...
    static constexpr bool in_hi(int e) { return e >= 8; }    // ... and the half of it
};
template <> struct PairMap<3> {  // 2-bit field at offset o with the extra bit below it: o = 2, 4, 6, 8
    static constexpr int n_pos = 4;
    static constexpr int lo(int k) { return k + 1; }
    static constexpr int hi(int k) { return (k + 9) & 15; }
    static constexpr int pos(int k) { return 2 * (k & 3) + 1; }
    static constexpr int k_of(int e) { return (e + 7) & 7; }
    static constexpr bool in_hi(int e) { return e == 0 || e >= 9; }
};
template <> struct PairMap<4> {  // nibbles at offset 0 and 4 of each half, directly and after a rotation by 8
    static constexpr int n_pos = 2;
    static constexpr int lo(int k) { return (k & 3) + 8 * (k >> 2); }
    static constexpr int hi(int k) { return lo(k) + 4; }
    static constexpr int pos(int k) { return 4 * (k & 1); }
    static constexpr int k_of(int e) { return (e & 3) + 4 * (e >> 3); }
    static constexpr bool in_hi(int e) { return ((e >> 2) & 1) != 0; }
};

template <int BITS> constexpr bool pair_map_consistent() {
    using M = PairMap<BITS>;
    for (int k = 0; k < 8; ++k)
        if (M::k_of(M::lo(k)) != k || M::in_hi(M::lo(k)) || M::k_of(M::hi(k)) != k || !M::in_hi(M::hi(k)) || M::pos(k) + BITS > 10) return false;
    return true;
}
static_assert(pair_map_consistent<2>() && pair_map_consistent<3>() && pair_map_consistent<4>(), "PairMap: element <-> (register, half) maps disagree");

// Every mask below is a literal of a two-operand `and` (see the note on instruction forms at the top), shifts go to
// the right wherever a plain shift does, and the one wrap-around that is needed (element 0 of the 3-bit layout) is a
// rotate.
// The 16 bits of the 1-bit plane spread so that the bit of element e sits at 2e - 1, directly below the element's 2-bit
// field of the 2-bit plane at 2e, 2e + 1 (element 0's bit wraps to bit 31).
FCV2_HD uint32_t spread_extra_bits16(uint32_t p1) {
    uint32_t x = and_lit<0x00FF00FFu>((p1 << 8) | p1);  // bit e -> 2e ...
    x = and_lit<0x0F0F0F0Fu>((x << 4) | x);
    x = and_lit<0x33333333u>((x << 2) | x);
    x = and_lit<0x55555555u>((x << 1) | x);
    return rotr32(x, 1);  // ... then turned right by one
}

// 3 bits: the pair registers from the 2-bit plane word and the spread extra bits S.
FCV2_HD void codes_pairs16_b3(uint32_t p2, uint32_t S, uint32_t (&Q)[8]) {
    // even elements: field at 4j, 4j + 1 from the plane, bit at 4j - 1 from S; odd elements: bit at 4j + 1 from S, field
    // at 4j + 2, 4j + 3 from the plane.  One bit-select each, with the same mask.
    const uint32_t M = vreg_const<0x33333333u>();
    const uint32_t We = bit_select(M, p2, S), Wo = bit_select(M, S, p2);
    const uint32_t We8 = rotr32(We, 8), Wo8 = Wo >> 8;  // elements 6, 8 / 14, 0 and 5, 7 / 13, 15 at the same four positions
    Q[0] = and_lit<0x000E000Eu>(Wo);   // elements 1, 9    at bit 1
    Q[1] = and_lit<0x00380038u>(We);   // elements 2, 10   at bit 3
    Q[2] = and_lit<0x00E000E0u>(Wo);   // elements 3, 11   at bit 5
    Q[3] = and_lit<0x03800380u>(We);   // elements 4, 12   at bit 7
    Q[4] = and_lit<0x000E000Eu>(Wo8);  // elements 5, 13
    Q[5] = and_lit<0x00380038u>(We8);  // elements 6, 14
    Q[6] = and_lit<0x00E000E0u>(Wo8);  // elements 7, 15
    Q[7] = and_lit<0x03800380u>(We8);  // elements 8, 0
}

template <int BITS> FCV2_HD void codes_pairs16(uint32_t p4a, uint32_t p4b, uint32_t p2, uint32_t p1, uint32_t (&Q)[8]) {
    if (BITS == 2) {
        const uint32_t B = p2 >> 10;  // element 5 at bit 0, element 13 at bit 16
        Q[0] = and_lit<0x00030003u>(p2);
        Q[1] = and_lit<0x000C000Cu>(p2);
        Q[2] = and_lit<0x00300030u>(p2);
        Q[3] = and_lit<0x00C000C0u>(p2);
        Q[4] = and_lit<0x03000300u>(p2);
        Q[5] = and_lit<0x00030003u>(B);
        Q[6] = and_lit<0x000C000Cu>(B);
        Q[7] = and_lit<0x00300030u>(B);
    } else if (BITS == 3) {
        codes_pairs16_b3(p2, spread_extra_bits16(p1), Q);
    } else {
        const uint32_t Ba = p4a >> 8, Bb = p4b >> 8;
        Q[0] = and_lit<0x000F000Fu>(p4a);
        Q[1] = and_lit<0x00F000F0u>(p4a);
        Q[2] = and_lit<0x000F000Fu>(Ba);
        Q[3] = and_lit<0x00F000F0u>(Ba);
        Q[4] = and_lit<0x000F000Fu>(p4b);
        Q[5] = and_lit<0x00F000F0u>(p4b);
        Q[6] = and_lit<0x000F000Fu>(Bb);
        Q[7] = and_lit<0x00F000F0u>(Bb);
    }
}

}  // namespace fcv2
