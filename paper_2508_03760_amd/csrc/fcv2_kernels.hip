// fcv2_kernels.hip -- HIP kernels and C ABI of libfcv2 for gfx950 (MI355X, wave64).
//
// Work decomposition: a lane owns EPL consecutive elements, a quantization group of G elements is owned by
// LPG = G/EPL neighbouring lanes, so group reductions are DPP butterflies inside a 16-lane row.  The kernels
// that stream a tensor once (quantize_pack, unpack_dequant, dispatch_quant) use EPL = 32 (64 bytes of bf16 per
// lane, LPG = 1..8): per-lane overheads are paid once per 32 elements, and a wave's tile of 2048 elements is moved
// with coalesced 16-byte accesses and transposed through LDS.  reduce_requant uses EPL = 16 (8 for groups of 32, so
// that a group still spans a quad): its accumulators and the values of one peer live in registers, and the spike
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
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <type_traits>

#include "../../include/fcv2.h"
#include "fcv2_bits.h"

namespace fcv2 {

struct Rec {  // section offsets of one packed record, relative to its first byte (records are < 4 GiB)
    uint32_t plane8, plane4, plane2, plane1, scale, zero, spike_val, spike_idx;
    uint32_t total;  // bytes of the record
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
    const int t = (int)threadIdx.x;
    tabs[t] = scale_table_pow(t);
    tabs[kScaleTablePow + t] = scale_table_thr(t);
    if (t < kScaleTablePow - 256) tabs[256 + t] = scale_table_pow(256 + t);
    if (t < kScaleTableThr - 256) tabs[kScaleTablePow + 256 + t] = scale_table_thr(256 + t);
    __syncthreads();
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

// Running two smallest values (m1 <= m2) of a stream.
__device__ __forceinline__ void push2(uint32_t& m1, uint32_t& m2, uint32_t c) {
    m2 = umed3(m1, m2, c);
    m1 = min(m1, c);
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
#pragma unroll
    for (int d = 0; d < EPL / 2; ++d) {
        typedef short short2v __attribute__((ext_vector_type(2)));
        const short2v sv = __builtin_bit_cast(short2v, w[d]);
        const uint32_t sign = __builtin_bit_cast(uint32_t, sv >> (short2v){15, 15});
        const uint32_t k = w[d] ^ (sign | 0x80008000u);  // two order keys
        uint32_t e0 = (k << 16) | (uint32_t)(2 * d), e1 = (k & 0xFFFF0000u) | (uint32_t)(2 * d + 1);
        FCV2_KEEP(e0);  // keeps each composite one shift-or / and-or instruction (no regrouping with the xor below)
        FCV2_KEEP(e1);
        const uint32_t f0 = e0 ^ 0xFFFF0000u, f1 = e1 ^ 0xFFFF0000u;  // inverted key: min finds the largest value
        if (d == 0) {
            a1 = min(e0, e1);
            a2 = max(e0, e1);
            b1 = min(f0, f1);
            b2 = max(f0, f1);
        } else if (SR) {
            push2(a1, a2, e0);
            push2(a1, a2, e1);
            push2(b1, b2, f0);
            push2(b1, b2, f1);
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
                cc = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_fminf(__fmul_rn(__fsub_rn(x, off), inv), (float)QMAX), b, cc);
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
template <int BITS, int EPL> __device__ __forceinline__ void store_planes(uint8_t* base, const Rec& r, uint32_t L,
                                                                           const uint32_t (&c)[EPL / 4]) {
    using P = Planes<BITS>;
    constexpr int U = EPL / 8;  // 8-element units
    if (P::w8) {
#pragma unroll
        for (int u = 0; u < U; u += 2) {
            uint8_t* at = base + (r.plane8 + (uint32_t)EPL * L + 8u * u);
            if (U >= 2)
                *reinterpret_cast<uint4*>(at) = make_uint4(c[2 * u], c[2 * u + 1], c[2 * u + 2], c[2 * u + 3]);
            else
                *reinterpret_cast<uint2*>(at) = make_uint2(c[0], c[1]);
        }
    }
    if (P::w4) {
        uint32_t q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = pack_plane4<P::sh4, BITS>(c[2 * u], c[2 * u + 1]);
        uint8_t* at = base + (r.plane4 + (uint32_t)(EPL / 2) * L);
        if (U == 4) *reinterpret_cast<uint4*>(at) = make_uint4(q[0], q[1], q[2], q[3]);
        if (U == 2) *reinterpret_cast<uint2*>(at) = make_uint2(q[0], q[1]);
        if (U == 1) *reinterpret_cast<uint32_t*>(at) = q[0];
    }
    if (P::w2) {
        uint32_t q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) q[u] = pack_plane2<P::sh2, BITS>(c[2 * u], c[2 * u + 1]) & 0xFFFFu;
        uint8_t* at = base + (r.plane2 + (uint32_t)(EPL / 4) * L);
        if (U == 4) *reinterpret_cast<uint2*>(at) = make_uint2(q[0] | (q[1] << 16), q[2] | (q[3] << 16));
        if (U == 2) *reinterpret_cast<uint32_t*>(at) = q[0] | (q[1] << 16);
        if (U == 1) *reinterpret_cast<uint16_t*>(at) = (uint16_t)q[0];
    }
    if (P::w1) {
        uint32_t q = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) q |= (pack_plane1<P::sh1, BITS>(c[2 * u], c[2 * u + 1]) & 0xFFu) << (8 * u);
        uint8_t* at = base + (r.plane1 + (uint32_t)(EPL / 8) * L);
        if (U == 4) *reinterpret_cast<uint32_t*>(at) = q;
        if (U == 2) *reinterpret_cast<uint16_t*>(at) = (uint16_t)q;
        if (U == 1) *at = (uint8_t)q;
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

// --- metadata fetched by quads (reduce_requant) ---------------------------------------------------------------
// Lane & 3 of every quad fetches one of the group's four metadata items (scale, zero, spike values, spike indices)
// as the aligned dword that holds it; quad broadcasts hand the four to every lane.  Address and byte selector of
// "its" item are computed once per lane and reused for every peer.
struct MetaOffsets {
    uint32_t at;   // aligned dword that holds the item
    uint32_t sel;  // byte selector (v_perm_b32) that moves the item to where its consumer wants it
};

template <int LPG, bool SR> __device__ __forceinline__ MetaOffsets meta_offsets(const Rec& r, uint32_t L, uint32_t mode) {
    const uint32_t g = L / LPG, item = L & 3u;
    const uint32_t msz = (mode == kMetaFp32) ? 4u : (mode == kMetaInt) ? 1u : 2u;
    uint32_t at = r.scale + msz * g;               // item 0, and every item when there are no spikes
    if (item == 1u) at = r.zero + msz * g;
    if (SR && item == 2u) at = r.spike_val + 4u * g;
    if (SR && item == 3u) at = r.spike_idx + 2u * g;
    MetaOffsets o;
    o.at = at & ~3u;
    // Selector bytes: 4 + k = byte k of the loaded dword, 0x0C = zero.
    const uint32_t b0 = 4u + (at & 3u), b1 = b0 + 1u;
    uint32_t sel = 0x07060504u;                                                      // fp32 items, spike values: as loaded
    if (mode == kMetaBf16) sel = 0x00000C0Cu | (b0 << 16) | (b1 << 24);              // bf16 -> the upper half: fp32 bits
    if (mode == kMetaInt) sel = 0x0C0C0C00u | b0;                                    // one byte -> the low byte
    if (SR && item == 2u) sel = 0x07060504u;
    if (SR && item == 3u) sel = 0x0C0C0000u | (b1 << 8) | b0;                        // two index bytes -> the low half
    o.sel = sel;
    return o;
}

template <bool SR, bool INT_META> __device__ __forceinline__ GroupMeta spread_meta(uint32_t raw, const MetaOffsets& o, const float* tabs) {
    const uint32_t val = __builtin_amdgcn_perm(raw, 0u, o.sel);
    GroupMeta m;
    const uint32_t sb = quad_bcast<0>(val), zb = quad_bcast<1>(val);
    if (INT_META) {  // Eq. 1 inverted: 2^(scale_int / 10), offset = -(zero * scale)
        m.s = tabs[(sb ^ 0x80u) + 1u];  // entry k + 129 of the table of 2^(k/10)
        m.lo = -__fmul_rn((float)zb, m.s);
    } else {
        m.s = u2f(sb);
        m.lo = u2f(zb);
    }
    m.raw_s = m.raw_z = 0;
    m.sv = SR ? quad_bcast<2>(val) : 0u;
    m.si = SR ? quad_bcast<3>(val) : 0u;
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
// and turned, through LDS, into 32 consecutive elements per lane.  Rows of 64 bytes are padded to 80 so that the
// 16-byte reads of 16 neighbouring lanes fall into different banks.
constexpr int kRowU4 = 5;  // uint4 per lane row: 4 of data + 1 of padding

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
        wave_lds[(P >> 2) * kRowU4 + (P & 3)] = t.piece[k];
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint4 v = wave_lds[lane * kRowU4 + k];
        w[4 * k] = v.x;
        w[4 * k + 1] = v.y;
        w[4 * k + 2] = v.z;
        w[4 * k + 3] = v.w;
    }
    wave_lds_sync();  // the next tile's writes must not overtake these reads
}

// Sender: persistent waves walk over the tiles; the next tile's loads are in flight while the current one is
// quantized, so memory and arithmetic overlap inside every wave.
template <int BITS, int LPG, bool SR, bool INT_META>
__global__ __launch_bounds__(kBlock) void k_quantize_pack_t(const uint4* __restrict__ x, uint32_t n_lanes, uint8_t* __restrict__ out,
                                                            Rec rec, uint32_t meta_mode_arg, uint32_t slice_lanes,
                                                            uint64_t record_stride) {
    // The integer metadata path is a compile-time variant here: its tables and extra live values would otherwise
    // cost the float formats a third of their registers (and with them two waves per SIMD).
    const uint32_t meta_mode = INT_META ? kMetaInt : (meta_mode_arg == kMetaFp32 ? kMetaFp32 : kMetaBf16);
    // The tensor may be cut into equal slices, each packed into a record of its own (records `record_stride` bytes
    // apart); slice_lanes is a multiple of 64 then, so a wave's tile lies in one slice.  One slice: slice_lanes = n_lanes.
    constexpr int EPL = kEplStream;
    __shared__ uint4 lds[kWaves][64 * kRowU4];
    __shared__ float tabs[kScaleTables];
    if (meta_mode == kMetaInt) fill_scale_tables(tabs);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));  // uniform: tiles are per wave
    const uint32_t lig = lane & (LPG - 1);
    const uint32_t n_tiles = (n_lanes + 63) / 64;
    const uint32_t stride = gridDim.x * kWaves;
    uint32_t tile = blockIdx.x * kWaves + wave;
    if (tile >= n_tiles) return;
    const uint32_t n_pieces = n_lanes * 4;
    auto process = [&](const TileIn& t, uint32_t tl) {
        uint32_t w[16];
        tile_transpose(t, lds[wave], lane, w);
        const uint32_t slice = (tl * 64) / slice_lanes;  // uniform
        const uint32_t L = tl * 64 + lane;
        if (L < n_lanes) {  // groups never straddle the end: whole groups are in or out together
            uint32_t c[EPL / 4];
            GroupMeta m;
            quantize_lane<BITS, EPL, LPG, SR>(w, lig, meta_mode, tabs, &lds[wave][lane * kRowU4], c, m);
            uint8_t* o = out + slice * record_stride;
            const uint32_t Lr = L - slice * slice_lanes;  // lane inside the record
            store_planes<BITS, EPL>(o, rec, Lr, c);
            if (lig == 0) store_meta<SR>(o, rec, Lr / LPG, m, meta_mode);
        }
    };
    // Two tiles are kept in flight per wave (two register sets, ping-pong, so loaded data is never moved); the
    // refill of a set is issued right after the tile that used it has been stored.  Loads are unconditional
    // (past the end they re-read the last tile): conditional ones would force full waits.
    const uint32_t last = n_tiles - 1;
    TileIn a = tile_load(x, (uint64_t)tile * 256, lane, n_pieces - tile * 256);
    uint32_t t1 = min(tile + stride, last);
    TileIn b = tile_load(x, (uint64_t)t1 * 256, lane, n_pieces - t1 * 256);
    while (true) {
        process(a, tile);
        uint32_t t2 = min(tile + 2 * stride, last);
        a = tile_load(x, (uint64_t)t2 * 256, lane, n_pieces - t2 * 256);
        tile += stride;
        if (tile >= n_tiles) break;
        process(b, tile);
        t2 = min(tile + 2 * stride, last);
        b = tile_load(x, (uint64_t)t2 * 256, lane, n_pieces - t2 * 256);
        tile += stride;
        if (tile >= n_tiles) break;
    }
}

// Receiver: 32 elements per lane; every lane reads its group's metadata itself.  The results go through LDS so that
// (a) the two spikes of a group are dropped into place by plain indexed LDS writes of the lanes that own their
// positions (Section 3.3: restored in place) and (b) the global stores are fully coalesced 16-byte pieces.
template <int BITS, int LPG, bool SR, bool OUT_FP32>
__global__ __launch_bounds__(kBlock) void k_unpack_dequant_t(PeerPtrs records, uint32_t slice_lanes, Rec rec, uint32_t n_lanes,
                                                             uint4* __restrict__ out, uint32_t meta_mode) {
    constexpr int EPL = kEplStream;
    constexpr int ROW = OUT_FP32 ? 9 : kRowU4;  // uint4 per lane row incl. one of padding
    constexpr int NP = OUT_FP32 ? 8 : 4;       // 16-byte pieces per lane
    __shared__ uint4 lds[kWaves][64 * ROW];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t lig = lane & (LPG - 1);
    const uint32_t tile = blockIdx.x * kWaves + wave;
    const uint32_t L = tile * 64 + lane;
    uint4* row = &lds[wave][lane * ROW];
    // The input may be several records, one per equal slice of the output (slice_lanes a multiple of 64 then).
    const uint32_t slice = (uint32_t)__builtin_amdgcn_readfirstlane((int)((tile * 64) / slice_lanes));
    if (L < n_lanes) {
        const uint8_t* __restrict__ in = records.base[slice];
        const uint32_t Lr = L - slice * slice_lanes;  // lane inside the record
        const uint32_t g = Lr / LPG;
        const RawPlanes<EPL> r = load_planes<BITS, EPL>(GlobalSrc{in}, rec, Lr);
        float s, lo;
        if (meta_mode == kMetaInt) {
            s = scale_of_int((int)(int8_t)in[rec.scale + g]);
            lo = -__fmul_rn((float)in[rec.zero + g], s);
        } else if (meta_mode == kMetaFp32) {
            s = *reinterpret_cast<const float*>(in + (rec.scale + 4u * g));
            lo = *reinterpret_cast<const float*>(in + (rec.zero + 4u * g));
        } else {
            s = u2f((uint32_t) * reinterpret_cast<const uint16_t*>(in + (rec.scale + 2u * g)) << 16);
            lo = u2f((uint32_t) * reinterpret_cast<const uint16_t*>(in + (rec.zero + 2u * g)) << 16);
        }
        uint32_t sv = 0, si = 0;
        if (SR) {
            sv = *reinterpret_cast<const uint32_t*>(in + (rec.spike_val + 4u * g));
            si = *reinterpret_cast<const uint16_t*>(in + (rec.spike_idx + 2u * g));
        }
#pragma unroll
        for (int u = 0; u < EPL / 8; ++u) {
            float q[8], v[8];
            unit_codes<BITS, EPL>(r, u, q);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = __fmaf_rn(q[j], s, lo);
            if (OUT_FP32) {
                row[2 * u] = make_uint4(f2u(v[0]), f2u(v[1]), f2u(v[2]), f2u(v[3]));
                row[2 * u + 1] = make_uint4(f2u(v[4]), f2u(v[5]), f2u(v[6]), f2u(v[7]));
            } else {
                row[u] = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
            }
        }
        if (SR) {
            const uint32_t relmin = (si & 0xFFu) - lig * (uint32_t)EPL, relmax = (si >> 8) - lig * (uint32_t)EPL;
            if (OUT_FP32) {
                u32a* o = reinterpret_cast<u32a*>(row);
                if (relmin < (uint32_t)EPL) o[relmin] = sv << 16;
                if (relmax < (uint32_t)EPL) o[relmax] = sv & 0xFFFF0000u;
            } else {
                u16a* o = reinterpret_cast<u16a*>(row);
                if (relmin < (uint32_t)EPL) o[relmin] = (uint16_t)sv;
                if (relmax < (uint32_t)EPL) o[relmax] = (uint16_t)(sv >> 16);
            }
        }
    }
    wave_lds_sync();
    const uint32_t n_pieces = n_lanes * NP;
    const uint32_t piece0 = tile * 64 * NP;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const uint32_t P = k * 64 + lane;
        if (piece0 + P < n_pieces) out[(uint64_t)piece0 + P] = lds[wave][(P / NP) * ROW + (P % NP)];
    }
}

// Local reduce step.  EPL = 16 elements per lane (8 for G = 32, so that a group still spans a whole quad).
//  - codes are unpacked into 16-bit halves and fed to v_fma_mix_f32 as fp16 denormals (q * 2^-24) against the
//    scale pre-multiplied by 2^24: the product is the same real number q * scale, the FMA rounds once, so the
//    result is bit-identical to fma(float(q), scale, lo) without a conversion instruction per element;
//  - the spike positions of every peer are patched through LDS: the (few) lanes that own a spike of this peer
//    park their values in a private LDS row, overwrite the spike slots with indexed writes and read the row
//    back -- a dynamic register index done by memory, paid only by the owners.
template <int BITS, int EPL>
__device__ __forceinline__ void dequant_mix(const RawPlanes<EPL>& r, float s, float lo, float (&v)[EPL]) {
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    using P = Planes<BITS>;
    if constexpr (EPL == 16 && BITS <= 4) {
        if (s < 0x1p+100f) {
            // Narrow codes are only masked in place (code << pos in each half); 2^-pos goes into the multiplier.
            using M = PairMap<BITS>;
            uint32_t Q[8];
            codes_pairs16<BITS>(P::w4 ? r.p4[0] : 0u, P::w4 ? r.p4[EPL / 8 - 1] : 0u, P::w2 ? r.p2[0] : 0u, P::w1 ? r.p1 : 0u, Q);
            float mult[9];
#pragma unroll
            for (int q = 0; q < 9; ++q) mult[q] = s * __builtin_ldexpf(1.0f, 24 - q);  // only the positions in use survive
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const half2v h = __builtin_bit_cast(half2v, Q[k]);
                v[M::lo(k)] = __builtin_fmaf((float)h.x, mult[M::pos(k)], lo);
                v[M::hi(k)] = __builtin_fmaf((float)h.y, mult[M::pos(k)], lo);
            }
            return;
        }
    }
    if (s < 0x1p+100f) {  // always, unless the data spans more than 2^100: then 2^24 * scale could overflow
        const float s24 = s * 0x1p+24f;
#pragma unroll
        for (int u = 0; u < EPL / 8; ++u) {
            uint32_t Q[4];
            const uint32_t p4 = P::w4 ? r.p4[u] : 0u;
            const uint32_t p2 = P::w2 ? ((r.p2[u >> 1] >> (16 * (u & 1))) & 0xFFFFu) : 0u;
            const uint32_t p1 = P::w1 ? ((r.p1 >> (8 * u)) & 0xFFu) : 0u;
            codes_pairs<BITS>(P::w8 ? r.p8[2 * u] : 0u, P::w8 ? r.p8[2 * u + 1] : 0u, p4, p2, p1, Q);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const half2v h = __builtin_bit_cast(half2v, Q[k]);
                v[8 * u + k] = __builtin_fmaf((float)h.x, s24, lo);
                v[8 * u + k + 4] = __builtin_fmaf((float)h.y, s24, lo);
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < EPL / 8; ++u) {
            float q[8];
            unit_codes<BITS, EPL>(r, u, q);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[8 * u + j] = __fmaf_rn(q[j], s, lo);
        }
    }
}

template <int EPL> __device__ __forceinline__ void patch_spikes(const GroupMeta& m, uint32_t lig, uint4* row, float (&v)[EPL]) {
    const uint32_t relmin = (m.si & 0xFFu) - lig * (uint32_t)EPL, relmax = (m.si >> 8) - lig * (uint32_t)EPL;
    if (relmin < (uint32_t)EPL || relmax < (uint32_t)EPL) {
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) row[i] = make_uint4(f2u(v[4 * i]), f2u(v[4 * i + 1]), f2u(v[4 * i + 2]), f2u(v[4 * i + 3]));
        u32a* o = reinterpret_cast<u32a*>(row);
        if (relmin < (uint32_t)EPL) o[relmin] = m.sv << 16;
        if (relmax < (uint32_t)EPL) o[relmax] = m.sv & 0xFFFF0000u;
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) {
            const uint4 a = row[i];
            v[4 * i] = u2f(a.x);
            v[4 * i + 1] = u2f(a.y);
            v[4 * i + 2] = u2f(a.z);
            v[4 * i + 3] = u2f(a.w);
        }
    }
}

template <int BITS, int EPL, int LPG, bool SR>
// Peers are taken two at a time (both peers' loads issued before either is decoded).  Every peer in flight costs
// about 15 registers; with two the kernel needs 65 to 74 and six or seven waves fit a SIMD, which measured faster
// than four peers in flight at four or five waves, and faster than one peer at eight.
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(6)))
void k_reduce_requant(PeerPtrs peers, int n_peers, uint32_t n_lanes, Rec rec_in,
                                                           uint8_t* __restrict__ out, Rec rec_out, float* __restrict__ sum_out,
                                                           uint32_t meta_mode_in, uint32_t meta_mode_out) {
    constexpr int CH = 2;  // peers in flight
    constexpr int ROW = EPL / 4 + 1;  // uint4 per private patch row, one of padding: conflict-free 16-byte accesses
    __shared__ uint4 lds[kBlock * ROW];
    __shared__ float tabs[kScaleTables];
    if (meta_mode_in == kMetaInt || meta_mode_out == kMetaInt) fill_scale_tables(tabs);
    const uint32_t L = blockIdx.x * kBlock + threadIdx.x;
    if (L >= n_lanes) return;
    const uint32_t lig = threadIdx.x & (LPG - 1);
    uint4* row = &lds[threadIdx.x * ROW];
    const MetaOffsets mo = meta_offsets<LPG, SR>(rec_in, L, meta_mode_in);
    // -0 is the identity of fp32 addition for every value including -0, so the chain below starts exactly at v_0
    float acc[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) acc[j] = -0.0f;
    // The peer loop exists twice, once per kind of metadata decoding, chosen by one uniform branch outside it.
    auto sum_peers = [&](auto int_meta) {
        constexpr bool INT_META = decltype(int_meta)::value;
        auto add_peer = [&](const RawPlanes<EPL>& r, uint32_t mraw) {
            const GroupMeta m = spread_meta<SR, INT_META>(mraw, mo, tabs);
            float v[EPL];
            dequant_mix<BITS, EPL>(r, m.s, m.lo, v);
            if (SR) patch_spikes<EPL>(m, lig, row, v);
#pragma unroll
            for (int j = 0; j < EPL; ++j) acc[j] = __fadd_rn(acc[j], v[j]);
        };
        int p = 0;
        // CH peers at a time: all loads first, so their latencies overlap
        for (; p + CH <= n_peers; p += CH) {
            RawPlanes<EPL> r[CH];
            uint32_t mraw[CH];
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const BufferSrc src = buffer_src(peers.base[p + i], rec_in.total);
                r[i] = load_planes<BITS, EPL>(src, rec_in, L);
                mraw[i] = ld32(src, mo.at);
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) add_peer(r[i], mraw[i]);
        }
        for (; p < n_peers; ++p) {
            const BufferSrc src = buffer_src(peers.base[p], rec_in.total);
            const RawPlanes<EPL> r = load_planes<BITS, EPL>(src, rec_in, L);
            const uint32_t mraw = ld32(src, mo.at);
            add_peer(r, mraw);
        }
    };
    if (meta_mode_in == kMetaInt)
        sum_peers(std::true_type{});
    else
        sum_peers(std::false_type{});
    if (sum_out) {
        float4* dst = reinterpret_cast<float4*>(sum_out) + (EPL / 4) * (uint64_t)L;
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) dst[i] = make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
    }
    uint32_t w[EPL / 2];
#pragma unroll
    for (int d = 0; d < EPL / 2; ++d) w[d] = pack_bf16(acc[2 * d], acc[2 * d + 1]);
    uint32_t c[EPL / 4];
    GroupMeta m;
    quantize_lane<BITS, EPL, LPG, SR>(w, lig, meta_mode_out, tabs, row, c, m);
    store_planes<BITS, EPL>(out, rec_out, L, c);
    if (lig == 0) store_meta<SR>(out, rec_out, L / LPG, m, meta_mode_out);
}

// The same step when the peers' bit width differs from the output's: the input width is a run-time value
// (one uniform switch per peer), the output width stays a template parameter.  Not pipelined; a compatibility
// path next to the specialised kernel above.
template <int BITS_OUT, int EPL, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_reduce_requant_mixed(PeerPtrs peers, int n_peers, uint32_t bits_in, uint32_t n_lanes,
                                                                 Rec rec_in, uint8_t* __restrict__ out, Rec rec_out,
                                                                 float* __restrict__ sum_out, uint32_t meta_mode_in,
                                                                 uint32_t meta_mode_out) {
    constexpr int ROW = EPL / 4 + 1;
    __shared__ uint4 lds[kBlock * ROW];
    __shared__ float tabs[kScaleTables];
    if (meta_mode_in == kMetaInt || meta_mode_out == kMetaInt) fill_scale_tables(tabs);
    const uint32_t L = blockIdx.x * kBlock + threadIdx.x;
    if (L >= n_lanes) return;
    const uint32_t lig = threadIdx.x & (LPG - 1);
    uint4* row = &lds[threadIdx.x * ROW];
    const MetaOffsets mo = meta_offsets<LPG, SR>(rec_in, L, meta_mode_in);
    float acc[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) acc[j] = -0.0f;
    for (int p = 0; p < n_peers; ++p) {
        const BufferSrc src = buffer_src(peers.base[p], rec_in.total);
        const uint32_t mraw = ld32(src, mo.at);
        const GroupMeta m = (meta_mode_in == kMetaInt) ? spread_meta<SR, true>(mraw, mo, tabs) : spread_meta<SR, false>(mraw, mo, tabs);
        float v[EPL];
        switch (bits_in) {
#define FCV2_CASE(B)                                                      \
    case B: {                                                             \
        const RawPlanes<EPL> r = load_planes<B, EPL>(src, rec_in, L);     \
        dequant_mix<B, EPL>(r, m.s, m.lo, v);                             \
        break;                                                            \
    }
            FCV2_CASE(2)
            FCV2_CASE(3)
            FCV2_CASE(4)
            FCV2_CASE(5)
            FCV2_CASE(6)
            FCV2_CASE(7)
            default:
                FCV2_CASE(8)
#undef FCV2_CASE
        }
        if (SR) patch_spikes<EPL>(m, lig, row, v);
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[j] = __fadd_rn(acc[j], v[j]);
    }
    if (sum_out) {
        float4* dst = reinterpret_cast<float4*>(sum_out) + (EPL / 4) * (uint64_t)L;
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) dst[i] = make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
    }
    uint32_t w[EPL / 2];
#pragma unroll
    for (int d = 0; d < EPL / 2; ++d) w[d] = pack_bf16(acc[2 * d], acc[2 * d + 1]);
    uint32_t c[EPL / 4];
    GroupMeta m;
    quantize_lane<BITS_OUT, EPL, LPG, SR>(w, lig, meta_mode_out, tabs, row, c, m);
    store_planes<BITS_OUT, EPL>(out, rec_out, L, c);
    if (lig == 0) store_meta<SR>(out, rec_out, L / LPG, m, meta_mode_out);
}

// ---- dispatch: stable counting sort of the routed copies by expert, then quantize-and-scatter ------------------------
constexpr int kChunk = 256;  // routed slots per block in the planning kernels

// Per-chunk histogram of expert ids.  hist[chunk][e].
__global__ __launch_bounds__(kChunk) void k_dispatch_count(const int32_t* __restrict__ ids, uint32_t n_slots, uint32_t E,
                                                           int32_t* __restrict__ hist) {
    extern __shared__ int32_t lds[];
    for (uint32_t e = threadIdx.x; e < E; e += kChunk) lds[e] = 0;
    __syncthreads();
    const uint32_t i = blockIdx.x * kChunk + threadIdx.x;
    if (i < n_slots) {
        const int32_t e = ids[i];
        if (e >= 0 && (uint32_t)e < E) atomicAdd(&lds[e], 1);  // integer counts: order does not matter
    }
    __syncthreads();
    for (uint32_t e = threadIdx.x; e < E; e += kChunk) hist[(uint64_t)blockIdx.x * E + e] = lds[e];
}

// Exclusive prefix sum of one value per thread over a block of 256 threads; *total gets the block sum.
__device__ __forceinline__ int32_t block_exclusive_scan_256(int32_t v, int32_t* lds4, int32_t* total) {
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t up = __shfl_up(inc, d);
        if ((int)lane >= d) inc += up;
    }
    if (lane == 63) lds4[wave] = inc;
    __syncthreads();
    int32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int32_t t = lds4[w];
        if ((uint32_t)w < wave) before += t;
        all += t;
    }
    *total = all;
    __syncthreads();
    return before + inc - v;
}

// One block per expert: exclusive prefix over the chunks, in place; totals[e] = count of expert e.
__global__ __launch_bounds__(256) void k_dispatch_scan_chunks(int32_t* __restrict__ hist, uint32_t n_chunks, uint32_t E,
                                                              int32_t* __restrict__ totals) {
    __shared__ int32_t lds4[4];
    const uint32_t e = blockIdx.x;
    const uint32_t per = (n_chunks + 255) / 256;  // consecutive chunks per thread
    const uint32_t c0 = threadIdx.x * per, c1 = min(c0 + per, n_chunks);
    int32_t s = 0;
    for (uint32_t c = c0; c < c1; ++c) s += hist[(uint64_t)c * E + e];
    int32_t total;
    int32_t run = block_exclusive_scan_256(s, lds4, &total);
    if (threadIdx.x == 0) totals[e] = total;
    for (uint32_t c = c0; c < c1; ++c) {
        const int32_t v = hist[(uint64_t)c * E + e];
        hist[(uint64_t)c * E + e] = run;
        run += v;
    }
}

// Destination row of every routed slot: expert start + copies in earlier chunks + copies earlier in this chunk.
// Every block derives the expert starts (exclusive scan of the totals) itself; block 0 also publishes them.
__global__ __launch_bounds__(kChunk) void k_dispatch_rank(const int32_t* __restrict__ ids, uint32_t n_slots, uint32_t E,
                                                          const int32_t* __restrict__ hist, const int32_t* __restrict__ totals,
                                                          int32_t* __restrict__ expert_offsets, int32_t* __restrict__ dest,
                                                          int32_t* __restrict__ row_src) {
    extern __shared__ int32_t lds[];  // [kChunk/64][E] copies of expert e in each wave of this chunk, then [E] expert starts
    __shared__ int32_t lds4[4];
    constexpr int kW = kChunk / 64;
    int32_t* start = lds + kW * E;
    for (uint32_t t = threadIdx.x; t < kW * E; t += kChunk) lds[t] = 0;
    {   // expert starts: consecutive experts per thread, block scan of the per-thread sums
        const uint32_t per = (E + kChunk - 1) / kChunk;
        const uint32_t e0 = threadIdx.x * per, e1 = min(e0 + per, E);
        int32_t s = 0;
        for (uint32_t e = e0; e < e1; ++e) s += totals[e];
        int32_t total;
        int32_t run = block_exclusive_scan_256(s, lds4, &total);
        for (uint32_t e = e0; e < e1; ++e) {
            start[e] = run;
            if (blockIdx.x == 0) expert_offsets[e] = run;
            run += totals[e];
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) expert_offsets[E] = total;
    }
    __syncthreads();
    const uint32_t i = blockIdx.x * kChunk + threadIdx.x;
    const uint32_t wave = threadIdx.x / 64, lane = threadIdx.x & 63;
    int32_t e = -1;
    if (i < n_slots) {
        e = ids[i];
        if (e < 0 || (uint32_t)e >= E) e = -1;
    }
    // stable rank inside the wave: lanes below me with the same expert
    uint32_t rank = 0;
    uint64_t todo = __ballot(e >= 0);
    while (todo) {  // one round per distinct expert id in the wave; every round clears at least one lane
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const int32_t el = __shfl(e, leader);
        const uint64_t same = __ballot(e == el);
        if (e == el) {
            rank = __popcll(same & ((1ull << lane) - 1ull));
            if ((int)lane == leader) lds[wave * E + el] = __popcll(same);
        }
        todo &= ~same;
    }
    __syncthreads();
    if (e >= 0) {
        uint32_t before = 0;
        for (uint32_t wv = 0; wv < wave; ++wv) before += lds[wv * E + e];
        const int32_t r = start[e] + hist[(uint64_t)blockIdx.x * E + e] + (int32_t)(before + rank);
        dest[i] = r;
        row_src[r] = (int32_t)i;
    } else if (i < n_slots) {
        dest[i] = -1;
    }
}

// Quantize every token once, store the packed row K times.  `rec` holds the row's section offsets (align 16).
// One wave tile = 2048 consecutive elements of x (rows are multiples of 32 elements, so a lane never straddles rows).
template <int BITS, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_dispatch_quant_t(const uint4* __restrict__ x, uint32_t n_lanes, uint32_t lanes_per_row,
                                                             uint32_t K, const int32_t* __restrict__ dest, uint8_t* __restrict__ send,
                                                             Rec rec, uint32_t row_bytes, uint32_t meta_mode) {
    constexpr int EPL = kEplStream;
    __shared__ uint4 lds[kWaves][64 * kRowU4];
    __shared__ float tabs[kScaleTables];
    if (meta_mode == kMetaInt) fill_scale_tables(tabs);
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t lig = lane & (LPG - 1);
    const uint32_t tile = blockIdx.x * kWaves + wave;
    if (tile * 64 >= n_lanes) return;
    const TileIn cur = tile_load(x, (uint64_t)tile * 256, lane, n_lanes * 4 - tile * 256);
    uint32_t w[16];
    tile_transpose(cur, lds[wave], lane, w);
    const uint32_t L = tile * 64 + lane;
    if (L >= n_lanes) return;
    const uint32_t t = L / lanes_per_row;
    const uint32_t r = L - t * lanes_per_row;  // lane inside the row
    uint32_t c[EPL / 4];
    GroupMeta m;
    quantize_lane<BITS, EPL, LPG, SR>(w, lig, meta_mode, tabs, &lds[wave][lane * kRowU4], c, m);
    const uint32_t g = r / LPG;
    // The send buffer is addressed with 32-bit offsets (checked on the host): a row's offset is one 24-bit multiply,
    // every store one add on top of per-lane offsets computed once.
    using P = Planes<BITS>;
    constexpr int U = EPL / 8;
    uint32_t q4[U], q2[U], q1 = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        q4[u] = P::w4 ? pack_plane4<P::sh4, BITS>(c[2 * u], c[2 * u + 1]) : 0u;
        q2[u] = P::w2 ? (pack_plane2<P::sh2, BITS>(c[2 * u], c[2 * u + 1]) & 0xFFFFu) : 0u;
        if (P::w1) q1 |= (pack_plane1<P::sh1, BITS>(c[2 * u], c[2 * u + 1]) & 0xFFu) << (8 * u);
    }
    const uint32_t o8 = rec.plane8 + 32u * r, o4 = rec.plane4 + 16u * r, o2 = rec.plane2 + 8u * r, o1 = rec.plane1 + 4u * r;
    const uint32_t msz = (meta_mode == kMetaFp32) ? 4u : (meta_mode == kMetaInt) ? 1u : 2u;
    const uint32_t os = rec.scale + msz * g, oz = rec.zero + msz * g, ov = rec.spike_val + 4u * g, oi = rec.spike_idx + 2u * g;
    for (uint32_t k0 = 0; k0 < K; k0 += 8) {
        int32_t rows[8];  // all destinations first: the loads overlap instead of queueing one behind the other
#pragma unroll
        for (int i = 0; i < 8; ++i) rows[i] = (k0 + i < K) ? dest[t * K + k0 + i] : -1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (rows[i] < 0) continue;
            const uint32_t ro = __umul24((uint32_t)rows[i], row_bytes);
            if (P::w8) {
                *reinterpret_cast<uint4*>(send + (ro + o8)) = make_uint4(c[0], c[1], c[2], c[3]);
                *reinterpret_cast<uint4*>(send + (ro + o8 + 16u)) = make_uint4(c[4], c[5], c[6], c[7]);
            }
            if (P::w4) *reinterpret_cast<uint4*>(send + (ro + o4)) = make_uint4(q4[0], q4[1], q4[2], q4[3]);
            if (P::w2) *reinterpret_cast<uint2*>(send + (ro + o2)) = make_uint2(q2[0] | (q2[1] << 16), q2[2] | (q2[3] << 16));
            if (P::w1) *reinterpret_cast<uint32_t*>(send + (ro + o1)) = q1;
            if (lig == 0) {
                if (meta_mode == kMetaInt) {
                    send[ro + os] = (uint8_t)m.raw_s;
                    send[ro + oz] = (uint8_t)m.raw_z;
                } else if (meta_mode == kMetaFp32) {
                    *reinterpret_cast<float*>(send + (ro + os)) = m.s;
                    *reinterpret_cast<float*>(send + (ro + oz)) = m.lo;
                } else {
                    *reinterpret_cast<uint16_t*>(send + (ro + os)) = (uint16_t)(f2u(m.s) >> 16);
                    *reinterpret_cast<uint16_t*>(send + (ro + oz)) = (uint16_t)(f2u(m.lo) >> 16);
                }
                if (SR) {
                    *reinterpret_cast<uint32_t*>(send + (ro + ov)) = m.sv;
                    *reinterpret_cast<uint16_t*>(send + (ro + oi)) = (uint16_t)m.si;
                }
            }
        }
    }
}

// Plain streaming copy (16 bytes per lane), used to measure the practical HBM ceiling next to the codec kernels.
__global__ __launch_bounds__(kBlock) void k_stream_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, uint64_t n16) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// ---- host side ---------------------------------------------------------------------------------------------------------
static bool fmt_supported(const fcv2_fmt_t* f) {
    if (f->bits < 2 || f->bits > 8) return false;
    if (f->group != 32 && f->group != 64 && f->group != 128 && f->group != 256) return false;
    if ((f->flags & ~(FCV2_F_SPIKE | FCV2_F_META_FP32 | FCV2_F_META_INT)) != 0) return false;
    return (f->flags & (FCV2_F_META_FP32 | FCV2_F_META_INT)) != (FCV2_F_META_FP32 | FCV2_F_META_INT);  // one or the other
}

static inline uint32_t meta_mode_of(const fcv2_fmt_t* f) {
    return (f->flags & FCV2_F_META_INT) ? kMetaInt : (f->flags & FCV2_F_META_FP32) ? kMetaFp32 : kMetaBf16;
}

static inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

static Rec rec_of(const fcv2_layout_t& l) {
    auto rel = [](uint64_t o) { return o == FCV2_ABSENT ? 0u : (uint32_t)o; };
    Rec r;
    r.plane8 = rel(l.off_plane8);
    r.plane4 = rel(l.off_plane4);
    r.plane2 = rel(l.off_plane2);
    r.plane1 = rel(l.off_plane1);
    r.scale = rel(l.off_scale);
    r.zero = rel(l.off_zero);
    r.spike_val = rel(l.off_spike_val);
    r.spike_idx = rel(l.off_spike_idx);
    r.total = (uint32_t)l.total_bytes;
    return r;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Calls F<BITS, G, SR>::run(args...) for the runtime format.
template <template <int, int, bool> class F, typename... A> static int by_format(const fcv2_fmt_t* f, A&&... a) {
    const bool sr = (f->flags & FCV2_F_SPIKE) != 0;
#define FCV2_CASE_G(B, G)                                                          \
    case G:                                                                        \
        return sr ? F<B, G, true>::run(a...) : F<B, G, false>::run(a...);
#define FCV2_CASE_B(B)                 \
    case B:                            \
        switch (f->group) {            \
            FCV2_CASE_G(B, 32)         \
            FCV2_CASE_G(B, 64)         \
            FCV2_CASE_G(B, 128)        \
            FCV2_CASE_G(B, 256)        \
        }                              \
        break;
    switch (f->bits) {
        FCV2_CASE_B(2)
        FCV2_CASE_B(3)
        FCV2_CASE_B(4)
        FCV2_CASE_B(5)
        FCV2_CASE_B(6)
        FCV2_CASE_B(7)
        FCV2_CASE_B(8)
    }
#undef FCV2_CASE_B
#undef FCV2_CASE_G
    return FCV2_ERR_UNSUPPORTED;
}

static inline int launch_status() { return hipGetLastError() == hipSuccess ? FCV2_OK : FCV2_ERR_LAUNCH; }

static inline unsigned grid_lanes(uint32_t n_lanes) { return (unsigned)((n_lanes + kBlock - 1) / kBlock); }

// Number of blocks of a persistent launch.  A compute unit holds 8 blocks of the quantize kernel (64 registers per
// lane, 20 KiB of LDS per block).  A tensor of at most that many tiles gets one wave per tile, all resident at once;
// a larger one gets 4 blocks per compute unit, each wave walking several tiles with the next loads in flight.
// FCV2_BLOCKS_PER_CU overrides the choice (for experiments).
static unsigned persistent_grid(uint32_t n_tiles) {
    static int cus = 0, forced = 0;
    if (cus == 0) {
        int dev = 0, n = 256;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 256;
        if (const char* e = getenv("FCV2_BLOCKS_PER_CU")) forced = atoi(e) > 0 ? atoi(e) : 0;
        cus = n > 0 ? n : 256;
    }
    const unsigned need = (n_tiles + kWaves - 1) / kWaves;
    const unsigned per_cu = forced ? (unsigned)forced : (need <= 8u * (unsigned)cus ? 8u : 4u);
    const unsigned blocks = per_cu * (unsigned)cus;
    return need < blocks ? need : blocks;
}

template <int BITS, int G, bool SR> struct LaunchQuantize {
    static int run(const void* x, uint64_t n, void* out, const Rec& rec, uint32_t meta_mode, uint32_t n_slices,
                   uint64_t record_stride, hipStream_t st) {
        constexpr int EPL = kEplStream;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        const uint32_t n_tiles = (n_lanes + 63) / 64;
        if (meta_mode == kMetaInt)
            hipLaunchKernelGGL((k_quantize_pack_t<BITS, G / EPL, SR, true>), dim3(persistent_grid(n_tiles)), dim3(kBlock), 0, st,
                               (const uint4*)x, n_lanes, (uint8_t*)out, rec, meta_mode, n_lanes / n_slices, record_stride);
        else
            hipLaunchKernelGGL((k_quantize_pack_t<BITS, G / EPL, SR, false>), dim3(persistent_grid(n_tiles)), dim3(kBlock), 0, st,
                               (const uint4*)x, n_lanes, (uint8_t*)out, rec, meta_mode, n_lanes / n_slices, record_stride);
        return launch_status();
    }
};
template <int BITS, int G, bool SR> struct LaunchUnpack {
    static int run(const PeerPtrs& records, uint32_t n_slices, const Rec& rec, uint64_t n, void* out, uint32_t out_fp32,
                   uint32_t meta_mode, hipStream_t st) {
        constexpr int EPL = kEplStream;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        if (out_fp32)
            hipLaunchKernelGGL((k_unpack_dequant_t<BITS, G / EPL, SR, true>), dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st,
                               records, n_lanes / n_slices, rec, n_lanes, (uint4*)out, meta_mode);
        else
            hipLaunchKernelGGL((k_unpack_dequant_t<BITS, G / EPL, SR, false>), dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st,
                               records, n_lanes / n_slices, rec, n_lanes, (uint4*)out, meta_mode);
        return launch_status();
    }
};
template <int BITS, int G, bool SR> struct LaunchReduce {
    static int run(const PeerPtrs& peers, int n_peers, uint64_t n, const Rec& rec_in, void* out, const Rec& rec_out,
                   float* sum_out, uint32_t mf_in, uint32_t mf_out, hipStream_t st) {
        constexpr int EPL = G >= 64 ? 16 : 8;  // 32 was measured: 180 VGPRs, two waves per SIMD, 15 % slower
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        hipLaunchKernelGGL((k_reduce_requant<BITS, EPL, G / EPL, SR>), dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st, peers,
                           n_peers, n_lanes, rec_in, (uint8_t*)out, rec_out, sum_out, mf_in, mf_out);
        return launch_status();
    }
};
template <int BITS, int G, bool SR> struct LaunchReduceMixed {  // BITS = output width
    static int run(const PeerPtrs& peers, int n_peers, uint32_t bits_in, uint64_t n, const Rec& rec_in, void* out,
                   const Rec& rec_out, float* sum_out, uint32_t mf_in, uint32_t mf_out, hipStream_t st) {
        constexpr int EPL = G >= 64 ? 16 : 8;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        hipLaunchKernelGGL((k_reduce_requant_mixed<BITS, EPL, G / EPL, SR>), dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st,
                           peers, n_peers, bits_in, n_lanes, rec_in, (uint8_t*)out, rec_out, sum_out, mf_in, mf_out);
        return launch_status();
    }
};
template <int BITS, int G, bool SR> struct LaunchDispatch {
    static int run(const void* x, uint64_t n, uint32_t H, uint32_t K, const int32_t* dest, uint8_t* send, const Rec& rec,
                   uint32_t row_bytes, uint32_t meta_mode, hipStream_t st) {
        constexpr int EPL = kEplStream;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        hipLaunchKernelGGL((k_dispatch_quant_t<BITS, G / EPL, SR>), dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st,
                           (const uint4*)x, n_lanes, H / EPL, K, dest, send, rec, row_bytes, meta_mode);
        return launch_status();
    }
};

struct DispatchWs {  // carving of the dispatch workspace
    uint32_t n_slots, n_chunks;
    size_t off_hist, off_totals, off_dest, bytes;
};
static DispatchWs dispatch_ws(uint32_t T, uint32_t K, uint32_t E) {
    DispatchWs w;
    w.n_slots = T * K;
    w.n_chunks = (w.n_slots + kChunk - 1) / kChunk;
    w.off_hist = 0;
    w.off_totals = round_up((size_t)w.n_chunks * E * 4, 256);
    w.off_dest = w.off_totals + round_up((size_t)E * 4, 256);
    w.bytes = w.off_dest + round_up((size_t)w.n_slots * 4, 256);
    return w;
}

}  // namespace fcv2

using namespace fcv2;

extern "C" {

int fcv2_version(void) { return 100; }

const char* fcv2_status_string(int s) {
    switch (s) {
        case FCV2_OK: return "ok";
        case FCV2_ERR_INVALID_ARG: return "invalid argument";
        case FCV2_ERR_UNSUPPORTED: return "unsupported format";
        case FCV2_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case FCV2_ERR_WORKSPACE: return "workspace too small";
        case FCV2_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

int fcv2_get_layout(uint64_t n, const fcv2_fmt_t* fmt, uint32_t align, fcv2_layout_t* out) {
    if (!fmt || !out) return FCV2_ERR_INVALID_ARG;
    if (!fmt_supported(fmt)) return FCV2_ERR_UNSUPPORTED;
    if (n == 0 || n % fmt->group != 0 || n % 8 != 0) return FCV2_ERR_INVALID_ARG;
    if (align == 0 || (align & (align - 1)) != 0) return FCV2_ERR_INVALID_ARG;
    const uint64_t ng = n / fmt->group;
    const uint64_t meta = (fmt->flags & FCV2_F_META_FP32) ? 4 : (fmt->flags & FCV2_F_META_INT) ? 1 : 2;
    const bool has8 = fmt->bits == 8, has4 = fmt->bits >= 4 && fmt->bits <= 7;
    const bool has2 = fmt->bits == 2 || fmt->bits == 3 || fmt->bits == 6 || fmt->bits == 7;
    const bool has1 = fmt->bits == 3 || fmt->bits == 5 || fmt->bits == 7;
    uint64_t off = 0;
    auto take = [&](bool present, uint64_t bytes) -> uint64_t {
        if (!present) return FCV2_ABSENT;
        off = round_up(off, align);
        const uint64_t at = off;
        off += bytes;
        return at;
    };
    out->n = n;
    out->n_groups = ng;
    out->off_plane8 = take(has8, n);
    out->off_plane4 = take(has4, n / 2);
    out->off_plane2 = take(has2, n / 4);
    out->off_plane1 = take(has1, n / 8);
    out->off_scale = take(true, ng * meta);
    out->off_zero = take(true, ng * meta);
    out->off_spike_val = take((fmt->flags & FCV2_F_SPIKE) != 0, ng * 4);
    out->off_spike_idx = take((fmt->flags & FCV2_F_SPIKE) != 0, ng * 2);
    out->total_bytes = round_up(off, align);  // the next record starts aligned too
    return FCV2_OK;
}

// Largest tensor the kernels index with 32-bit offsets: 2^31 elements (a 4 GiB bf16 tensor).
static const uint64_t kMaxElems = 1ull << 31;

// Slices of a two-step AllReduce payload: equal length, whole groups, whole 2048-element wave tiles.
static int check_slices(uint64_t n, uint32_t n_slices, const fcv2_fmt_t* fmt, fcv2_layout_t* slice_layout) {
    if (n_slices < 1 || n_slices > FCV2_MAX_PEERS || n == 0 || n % n_slices != 0) return FCV2_ERR_INVALID_ARG;
    const uint64_t len = n / n_slices;
    int rc = fcv2_get_layout(len, fmt, FCV2_TENSOR_ALIGN, slice_layout);
    if (rc != FCV2_OK) return rc;
    if (n_slices > 1 && len % 2048 != 0) return FCV2_ERR_INVALID_ARG;
    if (n > kMaxElems) return FCV2_ERR_UNSUPPORTED;
    return FCV2_OK;
}

int fcv2_quantize_pack_slices(const void* x, uint64_t n, uint32_t n_slices, const fcv2_fmt_t* fmt, void* packed,
                              uint64_t record_stride, void* stream) {
    if (!x || !packed || !fmt) return FCV2_ERR_INVALID_ARG;
    fcv2_layout_t l;
    int rc = check_slices(n, n_slices, fmt, &l);
    if (rc != FCV2_OK) return rc;
    if (n_slices > 1 && (record_stride < l.total_bytes || record_stride % FCV2_TENSOR_ALIGN != 0)) return FCV2_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(packed)) return FCV2_ERR_ALIGN;
    return by_format<LaunchQuantize>(fmt, x, n, packed, rec_of(l), meta_mode_of(fmt), n_slices,
                                     record_stride, (hipStream_t)stream);
}

int fcv2_quantize_pack(const void* x, uint64_t n, const fcv2_fmt_t* fmt, void* packed, void* stream) {
    return fcv2_quantize_pack_slices(x, n, 1, fmt, packed, 0, stream);
}

int fcv2_unpack_dequant_slices(const void* const* records, uint32_t n_slices, uint64_t n, const fcv2_fmt_t* fmt, void* out,
                               int out_dtype, void* stream) {
    if (!records || !out || !fmt) return FCV2_ERR_INVALID_ARG;
    if (out_dtype != FCV2_DT_BF16 && out_dtype != FCV2_DT_FP32) return FCV2_ERR_INVALID_ARG;
    fcv2_layout_t l;
    int rc = check_slices(n, n_slices, fmt, &l);
    if (rc != FCV2_OK) return rc;
    if (!aligned16(out)) return FCV2_ERR_ALIGN;
    PeerPtrs pp;
    for (uint32_t p = 0; p < FCV2_MAX_PEERS; ++p) {
        const void* ptr = records[p < n_slices ? p : 0];
        if (!ptr) return FCV2_ERR_INVALID_ARG;
        if (!aligned16(ptr)) return FCV2_ERR_ALIGN;
        pp.base[p] = (const uint8_t*)ptr;
    }
    return by_format<LaunchUnpack>(fmt, pp, n_slices, rec_of(l), n, out, (uint32_t)(out_dtype == FCV2_DT_FP32),
                                   meta_mode_of(fmt), (hipStream_t)stream);
}

int fcv2_unpack_dequant(const void* packed, uint64_t n, const fcv2_fmt_t* fmt, void* out, int out_dtype, void* stream) {
    const void* one[1] = {packed};
    if (!packed) return FCV2_ERR_INVALID_ARG;
    return fcv2_unpack_dequant_slices(one, 1, n, fmt, out, out_dtype, stream);
}

int fcv2_reduce_requant(const void* const* peers, int n_peers, uint64_t n, const fcv2_fmt_t* fmt_in, const fcv2_fmt_t* fmt_out,
                        void* packed_out, float* sum_out, void* stream) {
    if (!peers || !fmt_in || !fmt_out || !packed_out) return FCV2_ERR_INVALID_ARG;
    if (n_peers < 1 || n_peers > FCV2_MAX_PEERS) return FCV2_ERR_INVALID_ARG;
    fcv2_layout_t lin, lout;
    int rc = fcv2_get_layout(n, fmt_in, FCV2_TENSOR_ALIGN, &lin);
    if (rc != FCV2_OK) return rc;
    rc = fcv2_get_layout(n, fmt_out, FCV2_TENSOR_ALIGN, &lout);
    if (rc != FCV2_OK) return rc;
    if (n > kMaxElems) return FCV2_ERR_UNSUPPORTED;
    if (fmt_in->group != fmt_out->group || ((fmt_in->flags ^ fmt_out->flags) & FCV2_F_SPIKE) != 0)
        return FCV2_ERR_UNSUPPORTED;
    if (!aligned16(packed_out) || (sum_out && !aligned16(sum_out))) return FCV2_ERR_ALIGN;
    PeerPtrs pp;
    for (int p = 0; p < FCV2_MAX_PEERS; ++p) {
        const void* ptr = peers[p < n_peers ? p : 0];
        if (!ptr) return FCV2_ERR_INVALID_ARG;
        if (!aligned16(ptr)) return FCV2_ERR_ALIGN;
        pp.base[p] = (const uint8_t*)ptr;
    }
    const uint32_t mf_in = meta_mode_of(fmt_in);
    const uint32_t mf_out = meta_mode_of(fmt_out);
    if (fmt_in->bits != fmt_out->bits)
        return by_format<LaunchReduceMixed>(fmt_out, pp, n_peers, fmt_in->bits, n, rec_of(lin), packed_out, rec_of(lout), sum_out,
                                            mf_in, mf_out, (hipStream_t)stream);
    return by_format<LaunchReduce>(fmt_in, pp, n_peers, n, rec_of(lin), packed_out, rec_of(lout), sum_out, mf_in, mf_out,
                                   (hipStream_t)stream);
}

int fcv2_dispatch_workspace_bytes(uint32_t T, uint32_t K, uint32_t E, size_t* out) {
    if (!out || T == 0 || K == 0 || E == 0) return FCV2_ERR_INVALID_ARG;
    if ((uint64_t)T * K > 0x7FFFFFFFull) return FCV2_ERR_INVALID_ARG;
    if (E > 2048) return FCV2_ERR_UNSUPPORTED;  // per-wave expert counters and expert starts live in LDS (40 KiB at most)
    *out = dispatch_ws(T, K, E).bytes;
    return FCV2_OK;
}

int fcv2_dispatch_quant(const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E, const fcv2_fmt_t* fmt,
                        void* send, int32_t* expert_offsets, int32_t* row_src, void* ws, size_t ws_bytes, void* stream) {
    if (!x || !ids || !fmt || !send || !expert_offsets || !row_src || !ws) return FCV2_ERR_INVALID_ARG;
    size_t need = 0;
    int rc = fcv2_dispatch_workspace_bytes(T, K, E, &need);
    if (rc != FCV2_OK) return rc;
    fcv2_layout_t l;
    rc = fcv2_get_layout(H, fmt, FCV2_ROW_ALIGN, &l);
    if (rc != FCV2_OK) return rc;
    if ((uint64_t)T * H > kMaxElems) return FCV2_ERR_UNSUPPORTED;
    // rows are addressed with 24-bit row numbers and 32-bit byte offsets inside the send buffer
    if ((uint64_t)T * K >= (1u << 24) || l.total_bytes >= (1u << 24) || (uint64_t)T * K * l.total_bytes > 0xFFFFFFFFull)
        return FCV2_ERR_UNSUPPORTED;
    if (ws_bytes < need) return FCV2_ERR_WORKSPACE;
    if (!aligned16(x) || !aligned16(send) || !aligned16(ws) || ((uintptr_t)ids & 3u) || ((uintptr_t)expert_offsets & 3u) ||
        ((uintptr_t)row_src & 3u))
        return FCV2_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const DispatchWs w = dispatch_ws(T, K, E);
    int32_t* hist = (int32_t*)((uint8_t*)ws + w.off_hist);
    int32_t* totals = (int32_t*)((uint8_t*)ws + w.off_totals);
    int32_t* dest = (int32_t*)((uint8_t*)ws + w.off_dest);
    hipLaunchKernelGGL(k_dispatch_count, dim3(w.n_chunks), dim3(kChunk), E * 4, st, ids, w.n_slots, E, hist);
    hipLaunchKernelGGL(k_dispatch_scan_chunks, dim3(E), dim3(256), 0, st, hist, w.n_chunks, E, totals);
    hipLaunchKernelGGL(k_dispatch_rank, dim3(w.n_chunks), dim3(kChunk), (kChunk / 64 + 1) * E * 4, st, ids, w.n_slots, E, hist,
                       (const int32_t*)totals, expert_offsets, dest, row_src);
    if (launch_status() != FCV2_OK) return FCV2_ERR_LAUNCH;
    return by_format<LaunchDispatch>(fmt, x, (uint64_t)T * H, H, K, (const int32_t*)dest, (uint8_t*)send,
                                     rec_of(l), (uint32_t)l.total_bytes, meta_mode_of(fmt), st);
}

int fcv2_stream_copy(const void* src, void* dst, uint64_t bytes, void* stream) {
    if (!src || !dst || bytes == 0 || bytes % 16 != 0) return FCV2_ERR_INVALID_ARG;
    if (!aligned16(src) || !aligned16(dst)) return FCV2_ERR_ALIGN;
    const uint64_t n16 = bytes / 16;
    hipLaunchKernelGGL(k_stream_copy, dim3((unsigned)((n16 + kBlock - 1) / kBlock)), dim3(kBlock), 0, (hipStream_t)stream,
                       (const uint4*)src, (uint4*)dst, n16);
    return launch_status();
}

}  // extern "C"
