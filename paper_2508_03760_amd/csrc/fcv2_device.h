// fcv2_device.h -- device-side building blocks shared by the kernels of libfcv2 (gfx950, wave64).
//
// Work decomposition: a lane owns EPL consecutive elements, a quantization group of G elements is owned by
// LPG = G/EPL neighbouring lanes, so group reductions are DPP butterflies inside a 16-lane row.  The kernels
// that stream a tensor once (quantize_pack, unpack_dequant, dispatch_quant) use EPL = 32 (64 bytes of bf16 per
// lane, LPG = 1..8): per-lane overheads are paid once per 32 elements, and a wave's tile of 2048 elements is moved
// with coalesced 16-byte accesses and transposed through LDS.  reduce_requant uses EPL = 16 (a group
// is 2 to 16 lanes): its accumulators and the values of one peer live in registers, and the spike
// positions of every peer are patched through LDS.  The paper's own block shape (512 threads x 8 values,
// Section 4.1) was made for other hardware and is not followed.
//
// Arithmetic is fixed so that results can be compared bit for bit with an independent CPU implementation:
//   scale = (hi - lo) / qmax in fp32 (IEEE division), stored rounded up to bf16 unless FCV2_F_META_FP32;
//   inv = 1 / scale (IEEE division); code = clamp(rint((x - lo) * inv), 0, qmax), sub then mul, no FMA;
//   decode = fma(code, scale, lo); reduction = fp32 adds in peer order; bf16 rounding = nearest even.
//   With FCV2_F_META_INT (Section 3.3, Eq. 1) scale and zero are one byte each: the range is widened to contain 0,
//   scale_int = round(log2(scale) * 10), the decoded scale is 2^(scale_int / 10), zero = round(-lo / scale) as an
//   unsigned byte, the offset used by both sides is -(zero * scale), codes are clamped to [0, qmax].
// Compile with -ffp-contract=off.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/fcv2.h"
#include "../../include/fcv2_diag.h"
#include "fcv2_bits.h"

namespace fcv2 {

struct Rec {  // section offsets of one packed record, relative to its first byte (records are < 4 GiB)
    uint32_t plane8, plane4, plane2, plane1, scale, zero, spike_val, spike_idx;
    uint32_t total;  // bytes of the record
    uint32_t idx_bf16;  // spike positions stored as BF16 numbers, two bytes each (Table 4, first row), instead of bytes
};

struct PeerPtrs {
    const uint8_t* base[FCV2_MAX_PEERS];
};

struct GroupMeta {
    float s, lo;  // scale and offset as the receiver reconstructs them
    uint32_t sv;  // raw bf16 bits: min spike | max spike << 16
    uint32_t si;  // in-group positions: min | max << 8
    uint32_t raw_s, raw_z;  // integer metadata only: the scale_int byte and the zero byte
};

// How scale and zero are stored.
constexpr uint32_t kMetaBf16 = 0, kMetaFp32 = 1, kMetaInt = 2;

// Integer metadata: per-block LDS tables of 2^(k/10) and of the decision points of Eq. 1, one entry per code, so
// that coding and decoding a scale are table reads.  Called by all threads of a 256-thread block, before any of
// them leaves the kernel; tabs holds kScaleTablePow + kScaleTableThr floats.
constexpr int kScaleTables = kScaleTablePow + kScaleTableThr;
__device__ __forceinline__ void fill_scale_tables(float* tabs) {
    // a plain copy of the compile-time tables (515 floats): coalesced loads that depend on nothing, no arithmetic.
    // (Issuing a kernel's first tile loads before this copy, so that its latency runs under theirs, measured no faster.)
    const int t = (int)threadIdx.x;
    const float a = kScaleTablesInit.v[t], b = kScaleTablesInit.v[256 + t];
    const float c = kScaleTablesInit.v[t < kScaleTables - 512 ? 512 + t : 512];
    tabs[t] = a;
    tabs[256 + t] = b;
    if (t < kScaleTables - 512) tabs[512 + t] = c;
    __syncthreads();
}

// ---- streaming stores ---------------------------------------------------------------------------------------
// Output that is written once and not read again by the same kernel goes out with the non-temporal hint wherever a
// store instruction of the wave covers whole 128-byte lines.  Measured on the MI355X: a plain 16-byte-per-lane copy of
// 256 MiB takes 63 instead of 86 us (its source then stays in the last-level cache), unpack_dequant 16-25 % faster, the row copies of dispatch_quant 22 % faster.
// Stores that touch a few bytes per line (metadata written by one lane in four, 16-byte pieces 32 bytes apart) are
// slower with the hint and stay ordinary stores.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_stream(void* p, uint4 v) {
    const u32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void store_stream(void* p, uint2 v) {
    const u32x2 t = {v.x, v.y};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
}
__device__ __forceinline__ void store_stream(void* p, uint32_t v) { __builtin_nontemporal_store(v, reinterpret_cast<uint32_t*>(p)); }
__device__ __forceinline__ void store_stream(void* p, uint16_t v) { __builtin_nontemporal_store(v, reinterpret_cast<uint16_t*>(p)); }
__device__ __forceinline__ void store_stream(void* p, uint8_t v) { __builtin_nontemporal_store(v, reinterpret_cast<uint8_t*>(p)); }
__device__ __forceinline__ void store_stream(void* p, float v) { __builtin_nontemporal_store(v, reinterpret_cast<float*>(p)); }

// ---- block id -> tiles, per XCD -----------------------------------------------------------------------------------
// The hardware deals workgroups to the 8 XCDs round-robin by id, and every XCD has an L2 of its own.  Blocks that work
// on neighbouring tiles share cache lines of the metadata sections (a block's 32 groups are half a line of scales), so
// each XCD takes one contiguous eighth of the tiles: a shared line is then fetched into one L2, not two.  The grid is
// padded to a multiple of 8; ids past the last tile do nothing.
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ uint32_t xcd_tile_block(uint32_t block_id, uint32_t padded_grid) {
    return (block_id % kXcds) * (padded_grid / kXcds) + block_id / kXcds;
}

// ---- cross-lane helpers -------------------------------------------------------------------------------------
template <int CTRL> __device__ __forceinline__ uint32_t dpp(uint32_t v) {
    // old = identity of the unsigned minimum: the move folds into v_min_u32_dpp
    return (uint32_t)__builtin_amdgcn_update_dpp((int)0xFFFFFFFF, (int)v, CTRL, 0xF, 0xF, false);
}

// Value held by lane K of this lane's quad.
template <int K> __device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, K * 0x55, 0xF, 0xF, true);
}

// Views of LDS rows that are written as vectors and patched as scalars (or the other way round).
typedef uint32_t __attribute__((may_alias)) u32a;
typedef uint16_t __attribute__((may_alias)) u16a;

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ uint32_t umin3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r;
    asm("v_min3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Running two smallest values (m1 <= m2) of a stream, two new values at a time: the new second smallest is the smaller
// of the old one and the median of {m1, x, y} (m1 belongs to the three, so their median is the second smallest of the
// three; whatever is second smallest overall is either that or the old m2).  Three instructions for two values.
__device__ __forceinline__ void push2_pair(uint32_t& m1, uint32_t& m2, uint32_t x, uint32_t y) {
    const uint32_t t = umed3(m1, x, y);
    m1 = umin3(m1, x, y);
    m2 = min(m2, t);
}

// Two smallest values over the LPG lanes of a group (the lanes hold disjoint sets); all lanes get the result.
template <int CTRL> __device__ __forceinline__ void merge2_step(uint32_t& m1, uint32_t& m2) {
    const uint32_t p1lo = (uint32_t)__builtin_amdgcn_update_dpp((int)0xFFFFFFFF, (int)m1, CTRL, 0xF, 0xF, false);
    const uint32_t p1hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m1, CTRL, 0xF, 0xF, true);
    const uint32_t p2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m2, CTRL, 0xF, 0xF, true);
    const uint32_t t = max(m1, p1hi);
    m1 = min(m1, p1lo);
    m2 = min(min(t, m2), p2);
}
template <int LPG> __device__ __forceinline__ void group_min2(uint32_t& m1, uint32_t& m2) {
    if (LPG >= 2) merge2_step<0xB1>(m1, m2);
    if (LPG >= 4) merge2_step<0x4E>(m1, m2);
    if (LPG >= 8) merge2_step<0x141>(m1, m2);
    if (LPG >= 16) merge2_step<0x140>(m1, m2);
    if (LPG >= 32) {
        const uint32_t p1 = (uint32_t)__builtin_amdgcn_ds_swizzle((int)m1, 0x401F);  // lane ^ 16
        const uint32_t p2 = (uint32_t)__builtin_amdgcn_ds_swizzle((int)m2, 0x401F);
        const uint32_t t = max(m1, p1);
        m1 = min(m1, p1);
        m2 = min(min(t, m2), p2);
    }
}
template <int LPG> __device__ __forceinline__ uint32_t group_min(uint32_t v) {
    if (LPG >= 2) v = min(v, dpp<0xB1>(v));
    if (LPG >= 4) v = min(v, dpp<0x4E>(v));
    if (LPG >= 8) v = min(v, dpp<0x141>(v));
    if (LPG >= 16) v = min(v, dpp<0x140>(v));
    if (LPG >= 32) v = min(v, (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F));
    return v;
}

// 1 / s with IEEE rounding for s in [2^-64, 2^120]: hardware reciprocal (1 ulp) plus one Newton step.
// Checked on the MI355X against IEEE division for every fp32 value of that range: no mismatch.
__device__ __forceinline__ float rcp_newton(float s) {
    const float y0 = __builtin_amdgcn_rcpf(s);
    const float e = __fmaf_rn(-s, y0, 1.0f);
    return __fmaf_rn(e, y0, y0);
}

// Spike positions as the wire stores them with FCV2_F_IDX_BF16: the two positions (min | max << 8, each below 256) as two
// BF16 numbers (min in the low half).  Exact both ways: a position has at most 8 significant bits.
__device__ __forceinline__ uint32_t idx_pair_to_bf16(uint32_t si) {
    return (__float_as_uint((float)(si & 0xFFu)) >> 16) | (__float_as_uint((float)((si >> 8) & 0xFFu)) & 0xFFFF0000u);
}
// Back.  A well-formed record holds whole numbers below the group size here; anything else is a malformed record and
// outside the contract (values outside [0, 256) are read as position 255, fractions are cut off).
__device__ __forceinline__ uint32_t idx_pair_of_bf16(uint32_t raw) {
    const float a = __uint_as_float(raw << 16), b = __uint_as_float(raw & 0xFFFF0000u);
    const uint32_t ia = (a >= 0.0f && a < 256.0f) ? (uint32_t)a : 0xFFu, ib = (b >= 0.0f && b < 256.0f) ? (uint32_t)b : 0xFFu;
    return ia | (ib << 8);
}

// Two fp32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    typedef float float2v __attribute__((ext_vector_type(2)));
    typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((float2v){a, b}, bf2v));
}

// ---- encoder core: EPL consecutive bf16 values of this lane -> EPL codes (one per byte) + the group's metadata ----
// w[d] holds elements 2d (low half) and 2d+1 (high half).  lig = lane index inside the group (LPG = G / EPL lanes).
// row = this lane's private LDS scratch (at least EPL bytes, 16-byte aligned), free at the time of the call.
// Spike reserving (Section 3.3): the group's minimum and maximum are set aside (lowest index on ties, the
// maximum searched among the other positions) and the rest is quantized over [2nd smallest, 2nd largest]:
// the two smallest composites (key << 16 | position) and the two smallest of (~key << 16 | position) are
// tracked in one pass; the smallest of each gives a spike and its position, the second the new range.
template <int BITS, int EPL, int LPG, bool SR>
__device__ __forceinline__ void quantize_lane(const uint32_t (&w)[EPL / 2], uint32_t lig, uint32_t mode, const float* tabs, uint4* row,
                                              uint32_t (&c)[EPL / 4], GroupMeta& m) {
    const uint32_t lbase = lig * (uint32_t)EPL;
    uint32_t a1, a2, b1, b2;  // two smallest composites (a: minimum side, b: maximum side)
    const uint32_t key_flip = vreg_const<0x80008000u>();  // in a vector register: the three-register v_bitop3 is the cheap form
#pragma unroll
    for (int d = 0; d < EPL / 2; ++d) {
        typedef short short2v __attribute__((ext_vector_type(2)));
        const short2v sv = __builtin_bit_cast(short2v, w[d]);
        const uint32_t sign = __builtin_bit_cast(uint32_t, sv >> (short2v){15, 15});
        const uint32_t k = __builtin_amdgcn_bitop3_b32(sign, w[d], key_flip, 0x36);  // (sign | flip) ^ w: two order keys
        uint32_t e0 = (k << 16) | (uint32_t)(2 * d), e1 = (k & 0xFFFF0000u) | (uint32_t)(2 * d + 1);
        FCV2_KEEP(e0);  // keeps each composite one shift-or / and-or instruction (no regrouping with the xor below)
        FCV2_KEEP(e1);
        const uint32_t f0 = xor_lit<0xFFFF0000u>(e0), f1 = xor_lit<0xFFFF0000u>(e1);  // inverted key: min finds the largest value
        if (d == 0) {
            a1 = min(e0, e1);
            a2 = max(e0, e1);
            b1 = min(f0, f1);
            b2 = max(f0, f1);
        } else if (SR) {
            push2_pair(a1, a2, e0, e1);
            push2_pair(b1, b2, f0, f1);
        } else {
            a1 = min(a1, min(e0, e1));
            b1 = min(b1, min(f0, f1));
        }
    }
    a1 += lbase;
    b1 += lbase;
    uint32_t klo, khi, imin = 0xFFFFu, imax = 0xFFFFu;
    if (SR) {
        a2 += lbase;
        b2 += lbase;
        group_min2<LPG>(a1, a2);
        group_min2<LPG>(b1, b2);
        imin = a1 & 0xFFFFu;
        // a constant group: the first maximum is the minimum itself, take the next position
        imax = ((b1 & 0xFFFFu) == imin) ? (b2 & 0xFFFFu) : (b1 & 0xFFFFu);
        klo = a2 >> 16;
        khi = (~b2) >> 16;
        m.sv = bf16_of_key(a1 >> 16) | (bf16_of_key((~b1) >> 16) << 16);
        m.si = imin | (imax << 8);
    } else {
        a1 = group_min<LPG>(a1);
        b1 = group_min<LPG>(b1);
        klo = a1 >> 16;
        khi = (~b1) >> 16;
        m.sv = 0;
        m.si = 0;
    }
    const float lo = u2f(bf16_of_key(klo) << 16);
    const float hi = u2f(bf16_of_key(khi) << 16);
    constexpr int QMAX = (1 << BITS) - 1;
    float s, off, inv;
    uint32_t raw_s = 0, raw_z = 0;
    if (mode == kMetaInt) {
        // Eq. 1: byte-sized scale and zero-point over the range widened to contain 0
        const float lo0 = (lo < 0.0f) ? lo : 0.0f, hi0 = (hi > 0.0f) ? hi : 0.0f;
        const ScaleInt si = scale_int_from_tables(div_by_qmax<QMAX>(__fsub_rn(hi0, lo0)), tabs, tabs + kScaleTablePow);
        s = si.s;  // in [2^-12.8, 2^12.7]
        inv = rcp_newton(s);
        raw_z = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn(-lo0, inv), 0, 0u);  // nearest even, saturated to [0, 255]
        raw_s = (uint32_t)si.k & 0xFFu;
        off = -__fmul_rn((float)raw_z, s);
    } else {
        const float s32 = div_by_qmax<QMAX>(__fsub_rn(hi, lo));
        s = 1.0f;
        if (s32 >= 0x1p-64f) s = (mode == kMetaFp32) ? s32 : u2f(bf16_round_up_bits(f2u(s32)));
        if (!(s <= 0x1p+120f))
            inv = __fdiv_rn(1.0f, s);  // reciprocal near the denormal range, or an infinite scale
        else
            inv = rcp_newton(s);
        off = lo;
    }
    m.s = s;
    m.lo = off;
    m.raw_s = raw_s;
    m.raw_z = raw_z;

    // code = rint((x - off) * inv) clamped to [0, qmax].  v_cvt_pk_u8_f32 rounds to nearest even and saturates
    // to [0, 255] (NaN -> 0).  With float metadata (x - lo) * inv <= qmax * (1 + 2^-22) for every position outside
    // the spikes, so the conversion alone already is the clamped code; the minimum spike lands on 0 by itself, the
    // maximum spike's byte is cleared below.  With integer metadata the decoded scale may be up to 2^(1/20) below
    // the exact one, so the top is clamped explicitly, and the minimum spike's byte is cleared as well.
    if (BITS < 8 && mode == kMetaInt) {
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) {
            uint32_t cc = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int j = 4 * i + b;
                const float x = u2f((j & 1) ? (w[j >> 1] & 0xFFFF0000u) : (w[j >> 1] << 16));
                // median of (t, 0, qmax): the clamp, and 0 for a NaN (a sum over peers of which one decodes to NaN),
                // where a plain minimum with qmax would return qmax
                cc = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(__fmul_rn(__fsub_rn(x, off), inv), 0.0f, (float)QMAX), b, cc);
            }
            c[i] = cc;
        }
    } else {
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) {
            uint32_t cc = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int j = 4 * i + b;
                const float x = u2f((j & 1) ? (w[j >> 1] & 0xFFFF0000u) : (w[j >> 1] << 16));
                cc = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn(__fsub_rn(x, off), inv), b, cc);
            }
            c[i] = cc;
        }
    }
    if (SR) {
        // The codes at the spike positions are 0.  A position is a dynamic byte index into c[]: the owner lanes park
        // c[] in their private LDS row, clear the byte there and read the row back (a select per register would cost
        // three VALU operations per register for every lane).
        const uint32_t relmax = imax - lbase;  // position inside this lane, or >= EPL
        const uint32_t relmin = (mode == kMetaInt) ? imin - lbase : (uint32_t)EPL;
        if (relmax < (uint32_t)EPL || relmin < (uint32_t)EPL) {
            u32a* rw = reinterpret_cast<u32a*>(row);
            uint8_t* rb = reinterpret_cast<uint8_t*>(row);
            if (EPL >= 16) {
#pragma unroll
                for (int i = 0; i < EPL / 16; ++i) row[i] = make_uint4(c[4 * i], c[4 * i + 1], c[4 * i + 2], c[4 * i + 3]);
            } else {
#pragma unroll
                for (int i = 0; i < EPL / 4; ++i) rw[i] = c[i];
            }
            if (relmax < (uint32_t)EPL) rb[relmax] = 0;
            if (relmin < (uint32_t)EPL) rb[relmin] = 0;
            if (EPL >= 16) {
#pragma unroll
                for (int i = 0; i < EPL / 16; ++i) {
                    const uint4 v = row[i];
                    c[4 * i] = v.x;
                    c[4 * i + 1] = v.y;
                    c[4 * i + 2] = v.z;
                    c[4 * i + 3] = v.w;
                }
            } else {
#pragma unroll
                for (int i = 0; i < EPL / 4; ++i) c[i] = rw[i];
            }
        }
    }
}

// Store the planes of this lane's EPL codes.  L = lane index inside the record (element index / EPL).
// Plane stores: every store instruction of a wave covers consecutive bytes, and the record is on its way out of this
// GPU, so they carry the non-temporal hint.
template <int BITS, int EPL> __device__ __forceinline__ void store_planes(uint8_t* base, const Rec& r, uint32_t L,
                                                                           const uint32_t (&c)[EPL / 4]) {
    using P = Planes<BITS>;
    constexpr int U = EPL / 8;  // 8-element units
    if (P::w8) {
#pragma unroll
        for (int u = 0; u < U; u += 2) {
            uint8_t* at = base + (r.plane8 + (uint32_t)EPL * L + 8u * u);
            if (U >= 2)
                store_stream(at, make_uint4(c[2 * u], c[2 * u + 1], c[2 * u + 2], c[2 * u + 3]));
            else
                store_stream(at, make_uint2(c[0], c[1]));
        }
    }
    if (P::w4) {
        uint32_t q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = pack_plane4<P::sh4, BITS>(c[2 * u], c[2 * u + 1]);
        uint8_t* at = base + (r.plane4 + (uint32_t)(EPL / 2) * L);
        if (U == 4) store_stream(at, make_uint4(q[0], q[1], q[2], q[3]));
        if (U == 2) store_stream(at, make_uint2(q[0], q[1]));
        if (U == 1) store_stream(at, q[0]);
    }
    if (P::w2) {
        uint32_t q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = pack_plane2<P::sh2, BITS>(c[2 * u], c[2 * u + 1]);
        uint8_t* at = base + (r.plane2 + (uint32_t)(EPL / 4) * L);
        if (U == 4) store_stream(at, make_uint2(q[0] | (q[1] << 16), q[2] | (q[3] << 16)));
        if (U == 2) store_stream(at, q[0] | (q[1] << 16));
        if (U == 1) store_stream(at, (uint16_t)q[0]);
    }
    if (P::w1) {
        uint32_t q = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) q |= pack_plane1<P::sh1, BITS>(c[2 * u], c[2 * u + 1]) << (8 * u);
        uint8_t* at = base + (r.plane1 + (uint32_t)(EPL / 8) * L);
        if (U == 4) store_stream(at, q);
        if (U == 2) store_stream(at, (uint16_t)q);
        if (U == 1) store_stream(at, (uint8_t)q);
    }
}

template <bool SR> __device__ __forceinline__ void store_meta(uint8_t* base, const Rec& r, uint32_t g, const GroupMeta& m, uint32_t mode) {
    if (mode == kMetaInt) {
        base[r.scale + g] = (uint8_t)m.raw_s;
        base[r.zero + g] = (uint8_t)m.raw_z;
    } else if (mode == kMetaFp32) {
        *reinterpret_cast<float*>(base + (r.scale + 4u * g)) = m.s;
        *reinterpret_cast<float*>(base + (r.zero + 4u * g)) = m.lo;
    } else {
        *reinterpret_cast<uint16_t*>(base + (r.scale + 2u * g)) = (uint16_t)(f2u(m.s) >> 16);
        *reinterpret_cast<uint16_t*>(base + (r.zero + 2u * g)) = (uint16_t)(f2u(m.lo) >> 16);
    }
    if (SR) {
        *reinterpret_cast<uint32_t*>(base + (r.spike_val + 4u * g)) = m.sv;
        if (r.idx_bf16)
            *reinterpret_cast<uint32_t*>(base + (r.spike_idx + 4u * g)) = idx_pair_to_bf16(m.si);
        else
            *reinterpret_cast<uint16_t*>(base + (r.spike_idx + 2u * g)) = (uint16_t)m.si;
    }
}

// ---- decoder core ------------------------------------------------------------------------------------------------
// Address = uniform base + 32-bit lane offset.  Keeping the offset opaque at the point of use stops the compiler
// from widening it to 64 bits outside the peer loop, so every load keeps the scalar-base addressing form and
// needs no address arithmetic of its own.
__device__ __forceinline__ const uint8_t* at32(const uint8_t* __restrict__ base, uint32_t off) {
    asm volatile("" : "+v"(off));
    return base + off;
}

// Two ways to read a record.  GlobalSrc: plain global loads from base + offset.  BufferSrc: buffer loads through a
// resource descriptor (base, size) held in scalar registers; the 32-bit lane offset goes into the instruction as it
// is, so a loop over many records needs no per-record address arithmetic in vector registers, and reads past the
// record's size return 0 instead of touching memory.
struct GlobalSrc {
    const uint8_t* __restrict__ base;
};
struct BufferSrc {
    __amdgpu_buffer_rsrc_t rsrc;
};
__device__ __forceinline__ BufferSrc buffer_src(const uint8_t* base, uint32_t bytes) {
    BufferSrc b;
    b.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, (int)bytes, 0x00020000);  // raw 32-bit data
    return b;
}
__device__ __forceinline__ uint4 ld128(const GlobalSrc& s, uint32_t off) { return *reinterpret_cast<const uint4*>(at32(s.base, off)); }
__device__ __forceinline__ uint2 ld64(const GlobalSrc& s, uint32_t off) { return *reinterpret_cast<const uint2*>(at32(s.base, off)); }
__device__ __forceinline__ uint32_t ld32(const GlobalSrc& s, uint32_t off) { return *reinterpret_cast<const uint32_t*>(at32(s.base, off)); }
__device__ __forceinline__ uint32_t ld16(const GlobalSrc& s, uint32_t off) { return *reinterpret_cast<const uint16_t*>(at32(s.base, off)); }
__device__ __forceinline__ uint32_t ld8(const GlobalSrc& s, uint32_t off) { return *at32(s.base, off); }
__device__ __forceinline__ uint4 ld128(const BufferSrc& s, uint32_t off) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(s.rsrc, (int)off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 ld64(const BufferSrc& s, uint32_t off) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(s.rsrc, (int)off, 0, 0);
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint32_t ld32(const BufferSrc& s, uint32_t off) { return __builtin_amdgcn_raw_buffer_load_b32(s.rsrc, (int)off, 0, 0); }
__device__ __forceinline__ uint32_t ld16(const BufferSrc& s, uint32_t off) { return __builtin_amdgcn_raw_buffer_load_b16(s.rsrc, (int)off, 0, 0); }
__device__ __forceinline__ uint32_t ld8(const BufferSrc& s, uint32_t off) { return __builtin_amdgcn_raw_buffer_load_b8(s.rsrc, (int)off, 0, 0); }

// Plane pieces of one lane: EPL elements.
template <int EPL> struct RawPlanes {
    uint32_t p8[EPL / 4], p4[EPL / 8], p2[(EPL + 15) / 16], p1;
};

template <int BITS, int EPL, class SRC> __device__ __forceinline__ RawPlanes<EPL> load_planes(const SRC& src, const Rec& r, uint32_t L) {
    using P = Planes<BITS>;
    RawPlanes<EPL> o = {};
    if (P::w8) {
        const uint32_t at = r.plane8 + (uint32_t)EPL * L;
        if (EPL == 8) {
            const uint2 v = ld64(src, at);
            o.p8[0] = v.x;
            o.p8[1] = v.y;
        } else {
#pragma unroll
            for (int i = 0; i < EPL / 16; ++i) {
                const uint4 v = ld128(src, at + 16u * i);
                o.p8[4 * i] = v.x;
                o.p8[4 * i + 1] = v.y;
                o.p8[4 * i + 2] = v.z;
                o.p8[4 * i + 3] = v.w;
            }
        }
    }
    if (P::w4) {
        const uint32_t at = r.plane4 + (uint32_t)(EPL / 2) * L;
        if (EPL == 8) o.p4[0] = ld32(src, at);
        if (EPL == 16) {
            const uint2 v = ld64(src, at);
            o.p4[0] = v.x;
            o.p4[EPL / 8 - 1] = v.y;
        }
        if (EPL == 32) {
            const uint4 v = ld128(src, at);
            o.p4[0] = v.x;
            o.p4[1 % (EPL / 8)] = v.y;
            o.p4[2 % (EPL / 8)] = v.z;
            o.p4[3 % (EPL / 8)] = v.w;
        }
    }
    if (P::w2) {
        const uint32_t at = r.plane2 + (uint32_t)(EPL / 4) * L;
        if (EPL == 8) o.p2[0] = ld16(src, at);
        if (EPL == 16) o.p2[0] = ld32(src, at);
        if (EPL == 32) {
            const uint2 v = ld64(src, at);
            o.p2[0] = v.x;
            o.p2[(EPL + 15) / 16 - 1] = v.y;
        }
    }
    if (P::w1) {
        const uint32_t at = r.plane1 + (uint32_t)(EPL / 8) * L;
        if (EPL == 8) o.p1 = ld8(src, at);
        if (EPL == 16) o.p1 = ld16(src, at);
        if (EPL == 32) o.p1 = ld32(src, at);
    }
    return o;
}

// fp32 code values of unit u (8 elements) of the lane.
template <int BITS, int EPL> __device__ __forceinline__ void unit_codes(const RawPlanes<EPL>& r, int u, float (&q)[8]) {
    using P = Planes<BITS>;
    if (P::w8) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            q[j] = (float)((r.p8[2 * u] >> (8 * j)) & 0xFFu);
            q[j + 4] = (float)((r.p8[2 * u + 1] >> (8 * j)) & 0xFFu);
        }
    } else {
        uint32_t ev, od;
        const uint32_t p4 = P::w4 ? r.p4[u] : 0u;
        const uint32_t p2 = P::w2 ? ((r.p2[u >> 1] >> (16 * (u & 1))) & 0xFFFFu) : 0u;
        const uint32_t p1 = P::w1 ? ((r.p1 >> (8 * u)) & 0xFFu) : 0u;
        codes_even_odd<BITS>(p4, p2, p1, ev, od);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            q[2 * i] = (float)((ev >> (8 * i)) & 0xFFu);
            q[2 * i + 1] = (float)((od >> (8 * i)) & 0xFFu);
        }
    }
}

// --- metadata fetched cooperatively (reduce_requant) --------------------------------------------------------------
// The lanes of a group share the fetch of its four metadata items (scale, zero, spike values, spike indices), each
// read as the aligned dword that holds it and moved into place by one byte permute.  Groups of four or more lanes:
// lane & 3 of every quad fetches one item, quad broadcasts hand the four to every lane.  Groups of two lanes: the even
// lane fetches scale and spike values, the odd lane zero and spike indices, pair broadcasts hand them over.  Addresses
// and selectors are computed once per lane and reused for every peer.
struct MetaOffsets {
    uint32_t at, sel;    // aligned dword of the (first) item and its byte selector (v_perm_b32)
    uint32_t at2, sel2;  // second item, two-lane groups with spike reserving only
};

// kind: 0 scale, 1 zero, 2 spike values, 3 spike indices.  Selector bytes: 4 + k = byte k of the dword, 0x0C = zero.
__device__ __forceinline__ void meta_item(const Rec& r, uint32_t g, uint32_t mode, uint32_t kind, uint32_t& at_dword, uint32_t& sel) {
    const uint32_t msz = (mode == kMetaFp32) ? 4u : (mode == kMetaInt) ? 1u : 2u;
    uint32_t at = r.scale + msz * g;
    if (kind == 1u) at = r.zero + msz * g;
    if (kind == 2u) at = r.spike_val + 4u * g;
    if (kind == 3u) at = r.idx_bf16 ? r.spike_idx + 4u * g : r.spike_idx + 2u * g;
    const uint32_t b0 = 4u + (at & 3u), b1 = b0 + 1u;
    uint32_t s = 0x07060504u;                                                 // fp32 items, spike values: as loaded
    if (mode == kMetaBf16) s = 0x00000C0Cu | (b0 << 16) | (b1 << 24);         // bf16 -> the upper half: fp32 bits
    if (mode == kMetaInt) s = 0x0C0C0C00u | b0;                               // one byte -> the low byte
    if (kind == 2u) s = 0x07060504u;
    if (kind == 3u) s = r.idx_bf16 ? 0x07060504u : (0x0C0C0000u | (b1 << 8) | b0);  // two index bytes -> the low half (two BF16: as loaded)
    at_dword = at & ~3u;
    sel = s;
}

template <int LPG, bool SR> __device__ __forceinline__ MetaOffsets meta_offsets(const Rec& r, uint32_t L, uint32_t mode) {
    const uint32_t g = L / LPG;
    MetaOffsets o;
    if (LPG >= 4) {
        const uint32_t item = L & 3u;
        meta_item(r, g, mode, SR ? item : (item & 1u), o.at, o.sel);  // without spikes lanes 2, 3 repeat 0, 1
        o.at2 = o.at;
        o.sel2 = o.sel;
    } else {
        const uint32_t odd = L & 1u;
        meta_item(r, g, mode, odd, o.at, o.sel);
        meta_item(r, g, mode, SR ? 2u + odd : odd, o.at2, o.sel2);
    }
    return o;
}

// Value held by the even (ODD = 0) or odd lane of this lane's pair.
template <int ODD> __device__ __forceinline__ uint32_t pair_bcast(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ODD ? 0xF5 : 0xA0, 0xF, 0xF, true);  // quad_perm [1,1,3,3] / [0,0,2,2]
}

template <int LPG, bool SR, bool INT_META>
__device__ __forceinline__ GroupMeta spread_meta(uint32_t raw, uint32_t raw2, const MetaOffsets& o, const float* tabs, uint32_t idx_bf16) {
    const uint32_t val = __builtin_amdgcn_perm(raw, 0u, o.sel);
    GroupMeta m;
    uint32_t sb, zb;
    if (LPG >= 4) {
        sb = quad_bcast<0>(val);
        zb = quad_bcast<1>(val);
        m.sv = SR ? quad_bcast<2>(val) : 0u;
        m.si = SR ? quad_bcast<3>(val) : 0u;
    } else {
        sb = pair_bcast<0>(val);
        zb = pair_bcast<1>(val);
        const uint32_t val2 = SR ? __builtin_amdgcn_perm(raw2, 0u, o.sel2) : 0u;
        m.sv = SR ? pair_bcast<0>(val2) : 0u;
        m.si = SR ? pair_bcast<1>(val2) : 0u;
    }
    if (INT_META) {  // Eq. 1 inverted: 2^(scale_int / 10), offset = -(zero * scale)
        m.s = tabs[(sb ^ 0x80u) + 1u];  // entry k + 129 of the table of 2^(k/10)
        m.lo = -__fmul_rn((float)zb, m.s);
    } else {
        m.s = u2f(sb);
        m.lo = u2f(zb);
    }
    if (SR && idx_bf16) m.si = idx_pair_of_bf16(m.si);  // uniform branch: the positions travel as two BF16 numbers
    m.raw_s = m.raw_z = 0;
    return m;
}

// ---- kernels -------------------------------------------------------------------------------------------------------
constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kEplStream = 32;  // elements per lane in the kernels that stream a tensor once (64 bytes of bf16)

// Orders LDS traffic inside one wave: everything written before is visible to reads after (a wave's DS operations
// execute in order; this only stops the compiler from moving them across).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A wave's tile of 64 x 32 consecutive bf16 (4 KiB) is fetched with fully coalesced 16-byte loads (piece P = k*64 + lane)
// and turned, through LDS, into 32 consecutive elements per lane.  A lane's row is 64 bytes, four 16-byte slots, with
// no padding: slot q of row r lives at position q ^ ((r >> 1) & 3), so that the 16-byte reads of eight neighbouring
// lanes (two row parities x four slot positions) fall into eight different bank groups, and the writes of eight
// neighbouring lanes still cover two whole rows.  4 KiB per wave.
constexpr int kRowU4 = 4;  // uint4 per lane row
__device__ __forceinline__ uint32_t tile_slot(uint32_t row, uint32_t q) { return row * kRowU4 + (q ^ ((row >> 1) & 3u)); }

struct TileIn {
    uint4 piece[4];
};

__device__ __forceinline__ TileIn tile_load(const uint4* __restrict__ x, uint64_t tile_piece0, uint32_t lane, uint32_t pieces_left) {
    TileIn t;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        // pieces past the end re-read the last valid one: no branch, so the loads stay in one straight run and
        // the waits on them can be counted exactly (lanes that own such pieces never use them)
        const uint32_t P = min(k * 64 + lane, pieces_left - 1u);
        t.piece[k] = x[tile_piece0 + P];
    }
    return t;
}

__device__ __forceinline__ void tile_transpose(const TileIn& t, uint4* wave_lds, uint32_t lane, uint32_t (&w)[16]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t P = k * 64 + lane;
        wave_lds[tile_slot(P >> 2, P & 3)] = t.piece[k];
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint4 v = wave_lds[tile_slot(lane, k)];
        w[4 * k] = v.x;
        w[4 * k + 1] = v.y;
        w[4 * k + 2] = v.z;
        w[4 * k + 3] = v.w;
    }
    wave_lds_sync();  // the next tile's writes must not overtake these reads
}

}  // namespace fcv2
