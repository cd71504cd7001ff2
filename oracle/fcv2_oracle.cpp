// fcv2_oracle.cpp -- CPU oracle of the any-bit communication codec (FlashCommunication V2).
//
// TEST INFRASTRUCTURE ONLY: plain single-threaded C++17, one step after the other in the order the
// paper gives them, no blocking, no fusion, no SIMD.  Shares nothing with the HIP library.
// Build: g++ -std=c++17 -O2 -ffp-contract=off -fPIC -shared (see oracle/build.py).
//
// Readings taken where the paper is silent (each also listed in the design notes of this build):
//   * range after removing the spikes = min/max of the remaining G-2 values only (Section 3.3:
//     "shrunk range"); the zero written at a spike position does not take part;
//   * the code stored at a spike position is 0 (it is overwritten on decode);
//   * ties: lowest index; the max spike is searched among positions other than the min spike;
//   * order = total order on bf16 bit patterns (-0 < +0);
//   * rounding = round-half-to-even; scale = (hi-lo)/qmax in fp32, stored in bf16 rounded UP so that
//     qmax*scale still covers the range; the encoder quantizes with the stored scale; zero = lo
//     (a float offset, exact in bf16 because it is an input value);
//   * widest plane holds the most-significant bits ("first 4 bits" of Fig. 3); inside a plane byte
//     the element with the lowest index sits in the least-significant bits;
//   * spike indices are bytes (Section 3.3: "INT8"); with ORC_F_IDX_BF16 they are the positions written as BF16
//     numbers, two bytes each, which is the first row of Table 4 (2560 bytes for 4096 INT2 values in groups of 32);
//   * integer metadata (Eq. 1, Table 4 second row; flag ORC_F_META_INT): one signed byte
//     scale_int = round(log2(scale) * 10) clamped to [-128, 127], decoded as 2^(scale_int / 10) rounded to
//     fp32; one unsigned byte zero = the usual integer zero-point round(-lo / scale) over a range widened to
//     contain 0 (so it always fits the byte), decoded as the offset -(zero * scale); the encoder quantizes
//     with the decoded scale and offset, codes are clamped to [0, qmax].
#include "fcv2_oracle.h"

#include <cmath>
#include <cstring>
#include <vector>

namespace {

inline float bits_to_f32(uint32_t u) {
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}
inline uint32_t f32_to_bits(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return u;
}
inline float bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// Widths of the planes used for a b-bit code, widest (most significant) first.   (Section 3.2)
int plane_widths(uint32_t bits, int w[3]) {
    switch (bits) {
        case 2: w[0] = 2; return 1;
        case 3: w[0] = 2; w[1] = 1; return 2;
        case 4: w[0] = 4; return 1;
        case 5: w[0] = 4; w[1] = 1; return 2;
        case 6: w[0] = 4; w[1] = 2; return 2;
        case 7: w[0] = 4; w[1] = 2; w[2] = 1; return 3;
        case 8: w[0] = 8; return 1;
    }
    return 0;
}

bool fmt_ok(const orc_fmt* f) {
    return f && f->bits >= 2 && f->bits <= 8 && f->group >= 3 && f->group <= 256 &&
           (f->flags & ~(ORC_F_SPIKE | ORC_F_META_FP32 | ORC_F_META_INT | ORC_F_IDX_BF16)) == 0 &&
           (f->flags & (ORC_F_META_FP32 | ORC_F_META_INT)) != (ORC_F_META_FP32 | ORC_F_META_INT) &&
           (!(f->flags & ORC_F_IDX_BF16) || (f->flags & ORC_F_SPIKE));  // index width means something only with spikes
}

uint64_t plane_offset(const orc_layout& L, int width) {
    switch (width) {
        case 8: return L.off_plane8;
        case 4: return L.off_plane4;
        case 2: return L.off_plane2;
        default: return L.off_plane1;
    }
}

}  // namespace

extern "C" {

uint16_t orc_bf16_rne(float v) {
    uint32_t u = f32_to_bits(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN stays NaN
    uint32_t lsb = (u >> 16) & 1u;
    return (uint16_t)((u + 0x7FFFu + lsb) >> 16);
}

uint32_t orc_key(uint16_t u) { return (u & 0x8000u) ? ((uint32_t)(~u) & 0xFFFFu) : ((uint32_t)u | 0x8000u); }

// Table 4 counts: payload n*b/8 bytes; scale and zero one value per group each; one float value and
// one byte index per spike, two spikes per group.
int orc_get_layout(uint64_t n, const orc_fmt* fmt, uint32_t align, orc_layout* L) {
    if (!fmt_ok(fmt) || !L || n == 0 || align == 0 || n % fmt->group != 0 || n % 8 != 0) return ORC_ERR_ARG;
    L->n = n;
    L->n_groups = n / fmt->group;
    L->off_plane8 = L->off_plane4 = L->off_plane2 = L->off_plane1 = ORC_ABSENT;
    L->off_spike_val = L->off_spike_idx = ORC_ABSENT;
    int w[3];
    int np = plane_widths(fmt->bits, w);
    uint64_t off = 0;
    for (int p = 0; p < np; ++p) {
        off = round_up(off, align);
        if (w[p] == 8) L->off_plane8 = off;
        if (w[p] == 4) L->off_plane4 = off;
        if (w[p] == 2) L->off_plane2 = off;
        if (w[p] == 1) L->off_plane1 = off;
        off += n * (uint64_t)w[p] / 8;
    }
    uint64_t meta_elem = (fmt->flags & ORC_F_META_FP32) ? 4 : (fmt->flags & ORC_F_META_INT) ? 1 : 2;
    off = round_up(off, align);
    L->off_scale = off;
    off += L->n_groups * meta_elem;
    off = round_up(off, align);
    L->off_zero = off;
    off += L->n_groups * meta_elem;
    if (fmt->flags & ORC_F_SPIKE) {
        off = round_up(off, align);
        L->off_spike_val = off;
        off += L->n_groups * 2 * 2;
        off = round_up(off, align);
        L->off_spike_idx = off;
        off += L->n_groups * 2 * ((fmt->flags & ORC_F_IDX_BF16) ? 2 : 1);  // Table 4: indices in BF16 (first row) or INT8
    }
    L->total_bytes = round_up(off, align);  // records follow each other at aligned addresses
    return ORC_OK;
}

// Eq. 1 with theta = 10: the scale as one signed byte.  log2(0) = -inf lands on the lowest code, and so
// does a NaN.
int orc_scale_int(float scale) {
    if (!(scale > 0.0f)) return -128;
    const double t = std::nearbyint(std::log2((double)scale) * 10.0);
    return (int)std::fmin(std::fmax(t, -128.0), 127.0);
}

// The scale a receiver reconstructs from the byte: 2^(scale_int / theta), as an fp32 value.
float orc_scale_of_int(int scale_int) { return (float)std::exp2((double)scale_int / 10.0); }

// Integer metadata of one group from the range [lo, hi] that is to be quantized with `bits` bits: the range is
// widened to contain 0, the scale goes through Eq. 1, the zero-point is the rounded quotient -lo / scale (one
// unsigned byte).  s and zf are what the receiver reconstructs: scale and offset.
int orc_meta_int(float lo, float hi, uint32_t bits, int8_t* scale_int, uint8_t* zero_int, float* s, float* zf) {
    if (bits < 2 || bits > 8 || !scale_int || !zero_int || !s || !zf) return ORC_ERR_ARG;
    const int qmax = (1 << bits) - 1;
    const float lo0 = (lo < 0.0f) ? lo : 0.0f;
    const float hi0 = (hi > 0.0f) ? hi : 0.0f;
    const float s32 = (hi0 - lo0) / (float)qmax;
    const int k = orc_scale_int(s32);
    const float sd = orc_scale_of_int(k);
    const float inv = 1.0f / sd;
    const float tz = (-lo0) * inv;
    const int z = (tz >= 0.0f) ? (int)std::fmin(std::rint(tz), 255.0f) : 0;
    *scale_int = (int8_t)k;
    *zero_int = (uint8_t)z;
    *s = sd;
    *zf = -((float)z * sd);
    return ORC_OK;
}

}  // extern "C"

// One group.  Section 3.1 (asymmetric RTN per group) and Section 3.3 (spike reserving).  meta_int[2] receives the
// two metadata bytes when the format stores integer metadata.
static int quantize_group(const uint16_t* x, const orc_fmt* fmt, uint8_t* codes, float* scale, float* zero,
                          uint16_t* spike_val, uint8_t* spike_idx, uint8_t* meta_int) {
    if (!fmt_ok(fmt) || !x || !codes || !scale || !zero) return ORC_ERR_ARG;
    const int G = (int)fmt->group;
    const int qmax = (1 << fmt->bits) - 1;
    const bool sr = (fmt->flags & ORC_F_SPIKE) != 0;
    int imin = -1, imax = -1;
    if (sr) {
        if (!spike_val || !spike_idx) return ORC_ERR_ARG;
        // identify the minimum ... (lowest index on ties)
        imin = 0;
        for (int i = 1; i < G; ++i)
            if (orc_key(x[i]) < orc_key(x[imin])) imin = i;
        // ... and the maximum among the other positions (lowest index on ties)
        for (int i = 0; i < G; ++i) {
            if (i == imin) continue;
            if (imax < 0 || orc_key(x[i]) > orc_key(x[imax])) imax = i;
        }
        spike_val[0] = x[imin];
        spike_val[1] = x[imax];
        spike_idx[0] = (uint8_t)imin;
        spike_idx[1] = (uint8_t)imax;
    }
    // new minimum and maximum of what is left
    int ilo = -1, ihi = -1;
    for (int i = 0; i < G; ++i) {
        if (i == imin || i == imax) continue;
        if (ilo < 0 || orc_key(x[i]) < orc_key(x[ilo])) ilo = i;
        if (ihi < 0 || orc_key(x[i]) > orc_key(x[ihi])) ihi = i;
    }
    float lo = bf16_to_f32(x[ilo]);
    const float hi = bf16_to_f32(x[ihi]);
    float s;
    if (fmt->flags & ORC_F_META_INT) {
        int8_t k;
        uint8_t z;
        float zf;
        orc_meta_int(lo, hi, fmt->bits, &k, &z, &s, &zf);
        lo = zf;  // the offset the receiver will use
        meta_int[0] = (uint8_t)k;
        meta_int[1] = z;
    } else {
        const float s32 = (hi - lo) / (float)qmax;
        if (!(s32 >= 0x1p-64f)) {
            s = 1.0f;  // constant rest, vanishing range, or NaN
        } else if (fmt->flags & ORC_F_META_FP32) {
            s = s32;
        } else {
            s = bits_to_f32((f32_to_bits(s32) + 0xFFFFu) & 0xFFFF0000u);  // bf16, rounded up
        }
    }
    *scale = s;
    *zero = lo;
    const float inv = 1.0f / s;
    for (int i = 0; i < G; ++i) {
        if (i == imin || i == imax) {
            codes[i] = 0;
            continue;
        }
        const float d = bf16_to_f32(x[i]) - lo;
        const float t = d * inv;
        const float r = std::fmin(std::fmax(std::rint(t), 0.0f), (float)qmax);  // rint: half to even
        codes[i] = (uint8_t)(int)r;
    }
    return ORC_OK;
}

extern "C" {

int orc_quantize_group(const uint16_t* x, const orc_fmt* fmt, uint8_t* codes, float* scale, float* zero,
                       uint16_t* spike_val, uint8_t* spike_idx) {
    uint8_t meta_int[2];
    return quantize_group(x, fmt, codes, scale, zero, spike_val, spike_idx, meta_int);
}

// Bit splitting (Section 3.2): every plane is its own contiguous section.
int orc_split_pack(const uint8_t* codes, uint64_t n, const orc_fmt* fmt, uint32_t align, uint8_t* packed) {
    orc_layout L;
    if (!codes || !packed || orc_get_layout(n, fmt, align, &L) != ORC_OK) return ORC_ERR_ARG;
    int w[3];
    int np = plane_widths(fmt->bits, w);
    int shift = (int)fmt->bits;
    for (int p = 0; p < np; ++p) {
        shift -= w[p];  // this plane holds bits [shift, shift + w)
        uint8_t* dst = packed + plane_offset(L, w[p]);
        const uint64_t per_byte = 8 / w[p];
        const uint32_t mask = (1u << w[p]) - 1u;
        for (uint64_t j = 0; j < n / per_byte; ++j) {
            uint32_t byte = 0;
            for (uint64_t i = 0; i < per_byte; ++i) {
                uint32_t part = ((uint32_t)codes[j * per_byte + i] >> shift) & mask;
                byte |= part << (i * w[p]);
            }
            dst[j] = (uint8_t)byte;
        }
    }
    return ORC_OK;
}

int orc_unpack_codes(const uint8_t* packed, uint64_t n, const orc_fmt* fmt, uint32_t align, uint8_t* codes) {
    orc_layout L;
    if (!codes || !packed || orc_get_layout(n, fmt, align, &L) != ORC_OK) return ORC_ERR_ARG;
    int w[3];
    int np = plane_widths(fmt->bits, w);
    for (uint64_t e = 0; e < n; ++e) codes[e] = 0;
    int shift = (int)fmt->bits;
    for (int p = 0; p < np; ++p) {
        shift -= w[p];
        const uint8_t* src = packed + plane_offset(L, w[p]);
        const uint64_t per_byte = 8 / w[p];
        const uint32_t mask = (1u << w[p]) - 1u;
        for (uint64_t e = 0; e < n; ++e) {
            uint32_t part = ((uint32_t)src[e / per_byte] >> ((e % per_byte) * w[p])) & mask;
            codes[e] = (uint8_t)(codes[e] | (part << shift));
        }
    }
    return ORC_OK;
}

int orc_quantize_pack(const uint16_t* x, uint64_t n, const orc_fmt* fmt, uint32_t align, uint8_t* packed) {
    orc_layout L;
    if (!x || !packed || orc_get_layout(n, fmt, align, &L) != ORC_OK) return ORC_ERR_ARG;
    const uint32_t G = fmt->group;
    std::vector<uint8_t> codes(n);
    for (uint64_t g = 0; g < L.n_groups; ++g) {
        float s, z;
        uint16_t sv[2] = {0, 0};
        uint8_t si[2] = {0, 0};
        uint8_t mi[2] = {0, 0};
        int rc = quantize_group(x + g * G, fmt, codes.data() + g * G, &s, &z, sv, si, mi);
        if (rc != ORC_OK) return rc;
        if (fmt->flags & ORC_F_META_INT) {
            packed[L.off_scale + g] = mi[0];
            packed[L.off_zero + g] = mi[1];
        } else if (fmt->flags & ORC_F_META_FP32) {
            std::memcpy(packed + L.off_scale + 4 * g, &s, 4);
            std::memcpy(packed + L.off_zero + 4 * g, &z, 4);
        } else {
            // both are exactly representable in bf16 here: truncation loses nothing
            uint16_t sb = (uint16_t)(f32_to_bits(s) >> 16), zb = (uint16_t)(f32_to_bits(z) >> 16);
            std::memcpy(packed + L.off_scale + 2 * g, &sb, 2);
            std::memcpy(packed + L.off_zero + 2 * g, &zb, 2);
        }
        if (fmt->flags & ORC_F_SPIKE) {
            std::memcpy(packed + L.off_spike_val + 4 * g, sv, 4);
            if (fmt->flags & ORC_F_IDX_BF16) {
                // the position as a BF16 number (Table 4, first row): exact, positions are below 256
                const uint16_t ib[2] = {orc_bf16_rne((float)si[0]), orc_bf16_rne((float)si[1])};
                std::memcpy(packed + L.off_spike_idx + 4 * g, ib, 4);
            } else {
                std::memcpy(packed + L.off_spike_idx + 2 * g, si, 2);
            }
        }
    }
    return orc_split_pack(codes.data(), n, fmt, align, packed);
}

// Receiver side (Section 3.3): dequantize, then put the spikes back where they were.
// is_spike / raw_spike_bits (n entries each, or both null) report which positions were restored and
// the bf16 bit pattern put there, so a bf16 output can copy it unchanged.
static int decode_f32(const uint8_t* packed, uint64_t n, const orc_fmt* fmt, uint32_t align, float* v,
                      uint16_t* raw_spike_bits, uint8_t* is_spike) {
    orc_layout L;
    if (!packed || orc_get_layout(n, fmt, align, &L) != ORC_OK) return ORC_ERR_ARG;
    std::vector<uint8_t> codes(n);
    int rc = orc_unpack_codes(packed, n, fmt, align, codes.data());
    if (rc != ORC_OK) return rc;
    const uint32_t G = fmt->group;
    for (uint64_t g = 0; g < L.n_groups; ++g) {
        float s, z;
        if (fmt->flags & ORC_F_META_INT) {
            s = orc_scale_of_int((int)(int8_t)packed[L.off_scale + g]);
            z = -((float)packed[L.off_zero + g] * s);
        } else if (fmt->flags & ORC_F_META_FP32) {
            std::memcpy(&s, packed + L.off_scale + 4 * g, 4);
            std::memcpy(&z, packed + L.off_zero + 4 * g, 4);
        } else {
            uint16_t sb, zb;
            std::memcpy(&sb, packed + L.off_scale + 2 * g, 2);
            std::memcpy(&zb, packed + L.off_zero + 2 * g, 2);
            s = bf16_to_f32(sb);
            z = bf16_to_f32(zb);
        }
        for (uint32_t i = 0; i < G; ++i) {
            v[g * G + i] = std::fmaf((float)codes[g * G + i], s, z);
            if (is_spike) is_spike[g * G + i] = 0;
        }
        if (fmt->flags & ORC_F_SPIKE) {
            uint16_t sv[2];
            uint8_t si[2];
            std::memcpy(sv, packed + L.off_spike_val + 4 * g, 4);
            bool is_position[2] = {true, true};
            if (fmt->flags & ORC_F_IDX_BF16) {
                uint16_t ib[2];
                std::memcpy(ib, packed + L.off_spike_idx + 4 * g, 4);
                for (int k = 0; k < 2; ++k) {
                    const float pos = bf16_to_f32(ib[k]);
                    is_position[k] = pos >= 0.0f && pos < 256.0f && pos == std::floor(pos);
                    si[k] = is_position[k] ? (uint8_t)pos : 0;
                }
            } else {
                std::memcpy(si, packed + L.off_spike_idx + 2 * g, 2);
            }
            for (int k = 0; k < 2; ++k) {
                if (!is_position[k]) continue;  // malformed record: leave the dequantized value
                if (si[k] >= G) continue;  // malformed record: leave the dequantized value
                v[g * G + si[k]] = bf16_to_f32(sv[k]);
                if (is_spike) {
                    is_spike[g * G + si[k]] = 1;
                    raw_spike_bits[g * G + si[k]] = sv[k];
                }
            }
        }
    }
    return ORC_OK;
}

int orc_unpack_dequant(const uint8_t* packed, uint64_t n, const orc_fmt* fmt, uint32_t align, void* out,
                       int out_dtype) {
    if (!out || (out_dtype != ORC_DT_BF16 && out_dtype != ORC_DT_FP32)) return ORC_ERR_ARG;
    std::vector<float> v(n ? n : 1);
    std::vector<uint16_t> raw(n ? n : 1);
    std::vector<uint8_t> isp(n ? n : 1);
    int rc = decode_f32(packed, n, fmt, align, v.data(), raw.data(), isp.data());
    if (rc != ORC_OK) return rc;
    if (out_dtype == ORC_DT_FP32) {
        std::memcpy(out, v.data(), n * 4);
    } else {
        uint16_t* o = (uint16_t*)out;
        for (uint64_t e = 0; e < n; ++e) o[e] = isp[e] ? raw[e] : orc_bf16_rne(v[e]);
    }
    return ORC_OK;
}

// Local step of the two-step AllReduce (Sections 3.1, 3.4): dequantize every peer's chunk, add them
// up in fp32 in peer order, round the sum to bf16, quantize it again.
int orc_reduce_requant(const uint8_t* const* peers, int n_peers, uint64_t n, const orc_fmt* fmt_in,
                       const orc_fmt* fmt_out, uint32_t align, uint8_t* packed_out, float* sum_out) {
    if (!peers || n_peers < 1 || n_peers > 16 || !packed_out) return ORC_ERR_ARG;
    orc_layout Lin, Lout;
    if (orc_get_layout(n, fmt_in, align, &Lin) != ORC_OK || orc_get_layout(n, fmt_out, align, &Lout) != ORC_OK)
        return ORC_ERR_ARG;
    std::vector<float> acc(n), v(n);
    for (int p = 0; p < n_peers; ++p) {
        int rc = decode_f32(peers[p], n, fmt_in, align, v.data(), nullptr, nullptr);
        if (rc != ORC_OK) return rc;
        if (p == 0) {
            acc = v;
        } else {
            for (uint64_t e = 0; e < n; ++e) acc[e] = acc[e] + v[e];
        }
    }
    if (sum_out) std::memcpy(sum_out, acc.data(), n * 4);
    std::vector<uint16_t> y(n);
    for (uint64_t e = 0; e < n; ++e) y[e] = orc_bf16_rne(acc[e]);
    return orc_quantize_pack(y.data(), n, fmt_out, align, packed_out);
}

// Dispatch-only quantization (Section 3.1) with the routed copies grouped per expert: a stable
// counting sort of the (token, slot) pairs by expert id; every routed copy is the token's packed row.
int orc_dispatch_quant(const uint16_t* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E,
                       const orc_fmt* fmt, uint8_t* send_buf, int32_t* expert_offsets, int32_t* row_src) {
    orc_layout L;
    if (!x || !ids || !send_buf || !expert_offsets || !row_src || T == 0 || K == 0 || E == 0) return ORC_ERR_ARG;
    if (orc_get_layout(H, fmt, 16, &L) != ORC_OK) return ORC_ERR_ARG;
    const uint64_t row_bytes = L.total_bytes;
    std::vector<int64_t> count(E, 0);
    for (uint64_t i = 0; i < (uint64_t)T * K; ++i) {
        if (ids[i] == -1) continue;
        if (ids[i] < 0 || (uint32_t)ids[i] >= E) return ORC_ERR_ARG;
        count[ids[i]]++;
    }
    int64_t run = 0;
    for (uint32_t e = 0; e < E; ++e) {
        expert_offsets[e] = (int32_t)run;
        run += count[e];
    }
    expert_offsets[E] = (int32_t)run;
    std::vector<int64_t> next(E);
    for (uint32_t e = 0; e < E; ++e) next[e] = expert_offsets[e];
    std::vector<uint8_t> row(row_bytes);
    for (uint32_t t = 0; t < T; ++t) {
        std::memset(row.data(), 0, row_bytes);
        int rc = orc_quantize_pack(x + (uint64_t)t * H, H, fmt, 16, row.data());
        if (rc != ORC_OK) return rc;
        for (uint32_t k = 0; k < K; ++k) {
            int32_t e = ids[(uint64_t)t * K + k];
            if (e == -1) continue;
            int64_t r = next[e]++;
            row_src[r] = (int32_t)(t * K + k);
            std::memcpy(send_buf + (uint64_t)r * row_bytes, row.data(), row_bytes);
        }
    }
    return ORC_OK;
}

}  // extern "C"
