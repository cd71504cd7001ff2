// fcv2_kernels.hip -- HIP kernels and C ABI of libfcv2 for gfx950 (MI355X, wave64).
//
// Work decomposition shared by all kernels: one lane owns 8 consecutive elements (one 128-bit load of bf16),
// a quantization group of G elements is owned by LPG = G/8 neighbouring lanes (4, 8, 16 or 32), so group
// reductions are DPP butterflies inside a 16-lane row (plus one swizzle for G = 256).  The paper's own block
// shape (512 threads x 8 values, Section 4.1) was made for other hardware and is not followed.
//
// Arithmetic is fixed so that results can be compared bit for bit with an independent CPU implementation:
//   scale = (hi - lo) / qmax in fp32 (IEEE division), stored rounded up to bf16 unless FCV2_F_META_FP32;
//   inv = 1 / scale (IEEE division); code = clamp(rint((x - lo) * inv), 0, qmax), sub then mul, no FMA;
//   decode = fma(code, scale, lo); reduction = fp32 adds in peer order; bf16 rounding = nearest even.
// Compile with -ffp-contract=off.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fcv2.h"
#include "fcv2_bits.h"

namespace fcv2 {

struct Sections {  // device addresses of the sections of one packed record
    uint8_t* plane8;
    uint8_t* plane4;
    uint8_t* plane2;
    uint8_t* plane1;
    uint8_t* scale;
    uint8_t* zero;
    uint8_t* spike_val;
    uint8_t* spike_idx;
};

struct PeerArgs {
    Sections s[FCV2_MAX_PEERS];
};

struct GroupMeta {
    float s, lo;
    uint32_t sv;  // raw bf16 bits: min spike | max spike << 16
    uint32_t si;  // in-group positions: min | max << 8
};

// ---- cross-lane helpers -------------------------------------------------------------------------------------
template <int CTRL> __device__ __forceinline__ uint32_t dpp(uint32_t v) {
    // old = identity of the unsigned minimum: the move folds into v_min_u32_dpp
    return (uint32_t)__builtin_amdgcn_update_dpp((int)0xFFFFFFFF, (int)v, CTRL, 0xF, 0xF, false);
}

// Minimum over the LPG lanes of a group; every lane of the group gets the result.
template <int LPG> __device__ __forceinline__ uint32_t group_min(uint32_t v) {
    v = min(v, dpp<0xB1>(v));                   // quad_perm [1,0,3,2]
    v = min(v, dpp<0x4E>(v));                   // quad_perm [2,3,0,1]
    if (LPG >= 8) v = min(v, dpp<0x141>(v));    // row_half_mirror
    if (LPG >= 16) v = min(v, dpp<0x140>(v));   // row_mirror
    if (LPG >= 32) v = min(v, (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F));  // lane ^ 16
    return v;
}

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// 1 / s with IEEE rounding for a bf16-valued s in [2^-64, 2^120]: hardware reciprocal (1 ulp) plus one Newton
// step.  The quotient 2^k / m with an 8-bit significand m stays at least 2^-33 (relative) away from every
// rounding boundary, far more than the error left after the step, so the final rounding is the IEEE one.
__device__ __forceinline__ float rcp_of_bf16(float s) {
    const float y0 = __builtin_amdgcn_rcpf(s);
    const float e = __fmaf_rn(-s, y0, 1.0f);
    return __fmaf_rn(e, y0, y0);
}

// ---- encoder core: 8 bf16 values of this lane -> 8 codes (one per byte) + the group's metadata ----------------
// w[d] holds elements 2d (low half) and 2d+1 (high half).  lig = lane index inside the group.
// Spike reserving (Section 3.3): the group's minimum and maximum are set aside (lowest index on ties, the
// maximum searched among the other positions) and the rest is quantized over [2nd smallest, 2nd largest].
template <int BITS, int LPG, bool SR>
__device__ __forceinline__ void quantize8(const uint32_t (&w)[4], uint32_t lig, bool meta_fp32, uint32_t& c0,
                                          uint32_t& c1, GroupMeta& m) {
    constexpr float qmaxf = (float)((1 << BITS) - 1);
    const uint32_t lig8 = lig * 8u;

    // composite = order key << 16 | position: one unsigned min gives value and lowest index at once
    uint32_t cmin[8], cmax[8];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        typedef short short2v __attribute__((ext_vector_type(2)));
        short2v sv = __builtin_bit_cast(short2v, w[d]);
        uint32_t sign = __builtin_bit_cast(uint32_t, sv >> (short2v){15, 15});
        uint32_t k = w[d] ^ (sign | 0x80008000u);  // two order keys
        cmin[2 * d] = (k << 16) | (uint32_t)(2 * d);
        cmin[2 * d + 1] = (k & 0xFFFF0000u) | (uint32_t)(2 * d + 1);
        cmax[2 * d] = cmin[2 * d] ^ 0xFFFF0000u;  // inverted key: min finds the largest value
        cmax[2 * d + 1] = cmin[2 * d + 1] ^ 0xFFFF0000u;
    }
    uint32_t lmin = cmin[0], lmax = cmax[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) {
        lmin = min(lmin, cmin[j]);
        lmax = min(lmax, cmax[j]);
    }
    const uint32_t gmin = group_min<LPG>(lmin + lig8);
    const uint32_t gmax = group_min<LPG>(lmax + lig8);

    uint32_t klo, khi, imax = 0xFFFFu;
    if (SR) {
        // second smallest composite: everything except the one equal to the group minimum
        const uint32_t rmin = gmin - lig8 + 1u, rmax = gmax - lig8 + 1u;
        uint32_t l2min = cmin[0] - rmin, l2max = cmax[0] - rmax;  // the excluded entry wraps to 0xFFFFFFFF
#pragma unroll
        for (int j = 1; j < 8; ++j) {
            l2min = min(l2min, cmin[j] - rmin);
            l2max = min(l2max, cmax[j] - rmax);
        }
        const uint32_t g2min = group_min<LPG>(l2min + gmin + 1u);
        const uint32_t g2max = group_min<LPG>(l2max + gmax + 1u);
        const uint32_t imin = gmin & 0xFFFFu;
        // a constant group: the first maximum is the minimum itself, take the next position
        imax = ((gmax & 0xFFFFu) == imin) ? (g2max & 0xFFFFu) : (gmax & 0xFFFFu);
        klo = g2min >> 16;
        khi = (~g2max) >> 16;
        m.sv = bf16_of_key(gmin >> 16) | (bf16_of_key((~gmax) >> 16) << 16);
        m.si = imin | (imax << 8);
    } else {
        klo = gmin >> 16;
        khi = (~gmax) >> 16;
        m.sv = 0;
        m.si = 0;
    }
    const float lo = u2f(bf16_of_key(klo) << 16);
    const float hi = u2f(bf16_of_key(khi) << 16);
    const float s32 = div_by_qmax<(1 << BITS) - 1>(__fsub_rn(hi, lo));
    float s = 1.0f;
    if (s32 >= 0x1p-64f) s = meta_fp32 ? s32 : u2f(bf16_round_up_bits(f2u(s32)));
    float inv;
    if (meta_fp32 || !(s <= 0x1p+120f))
        inv = __fdiv_rn(1.0f, s);  // arbitrary significand, or a reciprocal near the denormal range
    else
        inv = rcp_of_bf16(s);
    m.s = s;
    m.lo = lo;

    c0 = 0;
    c1 = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float x = u2f((j & 1) ? (w[j >> 1] & 0xFFFF0000u) : (w[j >> 1] << 16));
        const float t = __fmul_rn(__fsub_rn(x, lo), inv);
        const float r = fminf(fmaxf(rintf(t), 0.0f), qmaxf);
        if (j < 4)
            c0 = __builtin_amdgcn_cvt_pk_u8_f32(r, j & 3, c0);
        else
            c1 = __builtin_amdgcn_cvt_pk_u8_f32(r, j & 3, c1);
    }
    if (SR) {
        // code 0 at the spike positions: the minimum already clamps to 0, clear the maximum's byte
        const uint32_t rel = imax - lig8;
        const uint32_t clr = ~(0xFFu << ((rel & 3u) * 8u));
        c0 &= (rel < 4u) ? clr : 0xFFFFFFFFu;
        c1 &= (rel - 4u < 4u) ? clr : 0xFFFFFFFFu;
    }
}

// Store the planes of this lane's 8 codes.  L = global lane index (element index / 8).
template <int BITS> __device__ __forceinline__ void store_planes(const Sections& o, uint64_t L, uint32_t c0, uint32_t c1) {
    using P = Planes<BITS>;
    if (P::w8) *reinterpret_cast<uint2*>(o.plane8 + 8 * L) = make_uint2(c0, c1);
    if (P::w4) *reinterpret_cast<uint32_t*>(o.plane4 + 4 * L) = pack_plane4<P::sh4, BITS>(c0, c1);
    if (P::w2) *reinterpret_cast<uint16_t*>(o.plane2 + 2 * L) = (uint16_t)pack_plane2<P::sh2, BITS>(c0, c1);
    if (P::w1) *(o.plane1 + L) = (uint8_t)pack_plane1<P::sh1, BITS>(c0, c1);
}

template <bool SR> __device__ __forceinline__ void store_meta(const Sections& o, uint64_t g, const GroupMeta& m, bool meta_fp32) {
    if (meta_fp32) {
        reinterpret_cast<float*>(o.scale)[g] = m.s;
        reinterpret_cast<float*>(o.zero)[g] = m.lo;
    } else {
        reinterpret_cast<uint16_t*>(o.scale)[g] = (uint16_t)(f2u(m.s) >> 16);
        reinterpret_cast<uint16_t*>(o.zero)[g] = (uint16_t)(f2u(m.lo) >> 16);
    }
    if (SR) {
        reinterpret_cast<uint32_t*>(o.spike_val)[g] = m.sv;
        reinterpret_cast<uint16_t*>(o.spike_idx)[g] = (uint16_t)m.si;
    }
}

// ---- decoder core: this lane's 8 elements of one packed record -> 8 fp32 values ---------------------------------
template <bool SR> __device__ __forceinline__ GroupMeta load_meta(const Sections& p, uint64_t g, bool meta_fp32) {
    GroupMeta m;
    if (meta_fp32) {
        m.s = reinterpret_cast<const float*>(p.scale)[g];
        m.lo = reinterpret_cast<const float*>(p.zero)[g];
    } else {
        m.s = u2f((uint32_t) reinterpret_cast<const uint16_t*>(p.scale)[g] << 16);
        m.lo = u2f((uint32_t) reinterpret_cast<const uint16_t*>(p.zero)[g] << 16);
    }
    if (SR) {
        m.sv = reinterpret_cast<const uint32_t*>(p.spike_val)[g];
        m.si = reinterpret_cast<const uint16_t*>(p.spike_idx)[g];
    } else {
        m.sv = 0;
        m.si = 0;
    }
    return m;
}

// v[j] = fma(code_j, scale, lo); spike positions get the stored float (Section 3.3: restored in place).
// spike_mask: bit j set where element j of this lane is a restored spike.
template <int BITS, bool SR>
__device__ __forceinline__ void dequant8(const Sections& p, uint64_t L, uint32_t lig, const GroupMeta& m, float (&v)[8],
                                         uint32_t& spike_mask, uint32_t (&spike_bits)[2]) {
    using P = Planes<BITS>;
    float q[8];
    if (P::w8) {
        const uint2 c = *reinterpret_cast<const uint2*>(p.plane8 + 8 * L);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            q[j] = (float)((c.x >> (8 * j)) & 0xFFu);
            q[j + 4] = (float)((c.y >> (8 * j)) & 0xFFu);
        }
    } else {
        uint32_t p4 = 0, p2 = 0, p1 = 0, ev, od;
        if (P::w4) p4 = *reinterpret_cast<const uint32_t*>(p.plane4 + 4 * L);
        if (P::w2) p2 = *reinterpret_cast<const uint16_t*>(p.plane2 + 2 * L);
        if (P::w1) p1 = *(p.plane1 + L);
        codes_even_odd<BITS>(p4, p2, p1, ev, od);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            q[2 * i] = (float)((ev >> (8 * i)) & 0xFFu);
            q[2 * i + 1] = (float)((od >> (8 * i)) & 0xFFu);
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __fmaf_rn(q[j], m.s, m.lo);
    spike_mask = 0;
    if (SR) {
        const uint32_t rel0 = (m.si & 0xFFu) - lig * 8u, rel1 = (m.si >> 8) - lig * 8u;
        const float f0 = u2f(m.sv << 16), f1 = u2f(m.sv & 0xFFFF0000u);
        spike_bits[0] = m.sv & 0xFFFFu;
        spike_bits[1] = m.sv >> 16;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[j] = (rel0 == (uint32_t)j) ? f0 : v[j];
            v[j] = (rel1 == (uint32_t)j) ? f1 : v[j];
        }
        spike_mask = (rel0 < 8u ? (1u << rel0) : 0u) | (rel1 < 8u ? (0x100u << rel1) : 0u);
    }
}

// ---- kernels -------------------------------------------------------------------------------------------------------
constexpr int kBlock = 256;

template <int BITS, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_quantize_pack(const uint4* __restrict__ x, uint64_t n_lanes, Sections out,
                                                          uint32_t meta_fp32) {
    const uint64_t L = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (L >= n_lanes) return;  // groups never straddle the end: whole groups leave together
    const uint32_t lig = threadIdx.x & (LPG - 1);
    const uint4 v = x[L];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t c0, c1;
    GroupMeta m;
    quantize8<BITS, LPG, SR>(w, lig, meta_fp32 != 0, c0, c1, m);
    store_planes<BITS>(out, L, c0, c1);
    if (lig == 0) store_meta<SR>(out, L / LPG, m, meta_fp32 != 0);
}

template <int BITS, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_unpack_dequant(Sections in, uint64_t n_lanes, void* __restrict__ out,
                                                           uint32_t out_fp32, uint32_t meta_fp32) {
    const uint64_t L = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (L >= n_lanes) return;
    const uint32_t lig = threadIdx.x & (LPG - 1);
    const GroupMeta m = load_meta<SR>(in, L / LPG, meta_fp32 != 0);
    float v[8];
    uint32_t mask, sb[2];
    dequant8<BITS, SR>(in, L, lig, m, v, mask, sb);
    if (out_fp32) {
        float4* o = reinterpret_cast<float4*>(out) + 2 * L;
        o[0] = make_float4(v[0], v[1], v[2], v[3]);
        o[1] = make_float4(v[4], v[5], v[6], v[7]);
    } else {
        uint32_t h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            h[j] = bf16_rne_bits(f2u(v[j]));
            if (SR) {  // spikes keep their stored bit pattern
                h[j] = (mask & (1u << j)) ? sb[0] : h[j];
                h[j] = (mask & (0x100u << j)) ? sb[1] : h[j];
            }
        }
        reinterpret_cast<uint4*>(out)[L] =
            make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
}

template <int BITS, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_reduce_requant(PeerArgs peers, int n_peers, uint64_t n_lanes, Sections out,
                                                           float* __restrict__ sum_out, uint32_t meta_fp32_in,
                                                           uint32_t meta_fp32_out) {
    const uint64_t L = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (L >= n_lanes) return;
    const uint32_t lig = threadIdx.x & (LPG - 1);
    const uint64_t g = L / LPG;
    float acc[8];
    for (int p = 0; p < n_peers; ++p) {
        const Sections& ps = peers.s[p];
        const GroupMeta m = load_meta<SR>(ps, g, meta_fp32_in != 0);
        float v[8];
        uint32_t mask, sb[2];
        dequant8<BITS, SR>(ps, L, lig, m, v, mask, sb);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = (p == 0) ? v[j] : __fadd_rn(acc[j], v[j]);
    }
    if (sum_out) {
        float4* o = reinterpret_cast<float4*>(sum_out) + 2 * L;
        o[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        o[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
    uint32_t w[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) w[d] = bf16_rne_bits(f2u(acc[2 * d])) | (bf16_rne_bits(f2u(acc[2 * d + 1])) << 16);
    uint32_t c0, c1;
    GroupMeta m;
    quantize8<BITS, LPG, SR>(w, lig, meta_fp32_out != 0, c0, c1, m);
    store_planes<BITS>(out, L, c0, c1);
    if (lig == 0) store_meta<SR>(out, g, m, meta_fp32_out != 0);
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

// One block per expert: exclusive prefix over the chunks, in place; totals[e] = count of expert e.
__global__ __launch_bounds__(256) void k_dispatch_scan_chunks(int32_t* __restrict__ hist, uint32_t n_chunks, uint32_t E,
                                                              int32_t* __restrict__ totals) {
    __shared__ int32_t part[256];
    const uint32_t e = blockIdx.x;
    const uint32_t per = (n_chunks + 255) / 256;  // consecutive chunks per thread
    const uint32_t c0 = threadIdx.x * per, c1 = min(c0 + per, n_chunks);
    int32_t s = 0;
    for (uint32_t c = c0; c < c1; ++c) s += hist[(uint64_t)c * E + e];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t run = 0;
        for (int t = 0; t < 256; ++t) {
            const int32_t v = part[t];
            part[t] = run;
            run += v;
        }
        totals[e] = run;
    }
    __syncthreads();
    int32_t run = part[threadIdx.x];
    for (uint32_t c = c0; c < c1; ++c) {
        const int32_t v = hist[(uint64_t)c * E + e];
        hist[(uint64_t)c * E + e] = run;
        run += v;
    }
}

// Exclusive scan of the expert totals into expert_offsets[E+1] (one block).
__global__ __launch_bounds__(256) void k_dispatch_scan_experts(const int32_t* __restrict__ totals, uint32_t E,
                                                               int32_t* __restrict__ expert_offsets) {
    __shared__ int32_t part[256];
    const uint32_t per = (E + 255) / 256;
    const uint32_t e0 = threadIdx.x * per, e1 = min(e0 + per, E);
    int32_t s = 0;
    for (uint32_t e = e0; e < e1; ++e) s += totals[e];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t run = 0;
        for (int t = 0; t < 256; ++t) {
            const int32_t v = part[t];
            part[t] = run;
            run += v;
        }
        expert_offsets[E] = run;
    }
    __syncthreads();
    int32_t run = part[threadIdx.x];
    for (uint32_t e = e0; e < e1; ++e) {
        expert_offsets[e] = run;
        run += totals[e];
    }
}

// Destination row of every routed slot: expert start + copies in earlier chunks + copies earlier in this chunk.
__global__ __launch_bounds__(kChunk) void k_dispatch_rank(const int32_t* __restrict__ ids, uint32_t n_slots, uint32_t E,
                                                          const int32_t* __restrict__ hist,
                                                          const int32_t* __restrict__ expert_offsets,
                                                          int32_t* __restrict__ dest, int32_t* __restrict__ row_src) {
    extern __shared__ int32_t lds[];  // [kChunk/64][E]: copies of expert e in each wave of this chunk
    constexpr int kWaves = kChunk / 64;
    for (uint32_t t = threadIdx.x; t < kWaves * E; t += kChunk) lds[t] = 0;
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
        const int32_t r = expert_offsets[e] + hist[(uint64_t)blockIdx.x * E + e] + (int32_t)(before + rank);
        dest[i] = r;
        row_src[r] = (int32_t)i;
    } else if (i < n_slots) {
        dest[i] = -1;
    }
}

// Quantize every token once, store the packed row K times.  Row sections are relative offsets (align 16).
struct RowLayout {
    uint32_t plane8, plane4, plane2, plane1, scale, zero, spike_val, spike_idx, row_bytes;
};

template <int BITS, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_dispatch_quant(const uint4* __restrict__ x, uint64_t n_lanes, uint32_t lanes_per_row,
                                                           uint32_t K, const int32_t* __restrict__ dest, uint8_t* __restrict__ send,
                                                           RowLayout rl, uint32_t meta_fp32) {
    const uint64_t L = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (L >= n_lanes) return;
    const uint32_t lig = threadIdx.x & (LPG - 1);
    const uint64_t t = L / lanes_per_row;
    const uint32_t r = (uint32_t)(L - t * lanes_per_row);  // lane inside the row
    const uint4 v = x[L];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t c0, c1;
    GroupMeta m;
    quantize8<BITS, LPG, SR>(w, lig, meta_fp32 != 0, c0, c1, m);
    for (uint32_t k = 0; k < K; ++k) {
        const int32_t row = dest[t * K + k];
        if (row < 0) continue;
        uint8_t* base = send + (uint64_t)row * rl.row_bytes;
        Sections o;
        o.plane8 = base + rl.plane8;
        o.plane4 = base + rl.plane4;
        o.plane2 = base + rl.plane2;
        o.plane1 = base + rl.plane1;
        o.scale = base + rl.scale;
        o.zero = base + rl.zero;
        o.spike_val = base + rl.spike_val;
        o.spike_idx = base + rl.spike_idx;
        store_planes<BITS>(o, r, c0, c1);
        if (lig == 0) store_meta<SR>(o, r / LPG, m, meta_fp32 != 0);
    }
}

// ---- host side ---------------------------------------------------------------------------------------------------------
static bool fmt_supported(const fcv2_fmt_t* f) {
    if (f->bits < 2 || f->bits > 8) return false;
    if (f->group != 32 && f->group != 64 && f->group != 128 && f->group != 256) return false;
    return (f->flags & ~(FCV2_F_SPIKE | FCV2_F_META_FP32)) == 0;
}

static inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

static Sections sections_of(const void* base, const fcv2_layout_t& l) {
    uint8_t* b = (uint8_t*)base;
    Sections s;
    s.plane8 = l.off_plane8 == FCV2_ABSENT ? nullptr : b + l.off_plane8;
    s.plane4 = l.off_plane4 == FCV2_ABSENT ? nullptr : b + l.off_plane4;
    s.plane2 = l.off_plane2 == FCV2_ABSENT ? nullptr : b + l.off_plane2;
    s.plane1 = l.off_plane1 == FCV2_ABSENT ? nullptr : b + l.off_plane1;
    s.scale = b + l.off_scale;
    s.zero = b + l.off_zero;
    s.spike_val = l.off_spike_val == FCV2_ABSENT ? nullptr : b + l.off_spike_val;
    s.spike_idx = l.off_spike_idx == FCV2_ABSENT ? nullptr : b + l.off_spike_idx;
    return s;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Calls F<BITS, LPG, SR>::run(args...) for the runtime format.
template <template <int, int, bool> class F, typename... A> static int by_format(const fcv2_fmt_t* f, A&&... a) {
    const bool sr = (f->flags & FCV2_F_SPIKE) != 0;
#define FCV2_CASE_G(B, G)                                                          \
    case G:                                                                        \
        return sr ? F<B, G / 8, true>::run(a...) : F<B, G / 8, false>::run(a...);
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
static inline unsigned grid_for(uint64_t n_lanes) { return (unsigned)((n_lanes + kBlock - 1) / kBlock); }

template <int BITS, int LPG, bool SR> struct LaunchQuantize {
    static int run(const void* x, uint64_t n_lanes, const Sections& out, uint32_t meta_fp32, hipStream_t st) {
        hipLaunchKernelGGL((k_quantize_pack<BITS, LPG, SR>), dim3(grid_for(n_lanes)), dim3(kBlock), 0, st, (const uint4*)x,
                           n_lanes, out, meta_fp32);
        return launch_status();
    }
};
template <int BITS, int LPG, bool SR> struct LaunchUnpack {
    static int run(const Sections& in, uint64_t n_lanes, void* out, uint32_t out_fp32, uint32_t meta_fp32, hipStream_t st) {
        hipLaunchKernelGGL((k_unpack_dequant<BITS, LPG, SR>), dim3(grid_for(n_lanes)), dim3(kBlock), 0, st, in, n_lanes, out,
                           out_fp32, meta_fp32);
        return launch_status();
    }
};
template <int BITS, int LPG, bool SR> struct LaunchReduce {
    static int run(const PeerArgs& peers, int n_peers, uint64_t n_lanes, const Sections& out, float* sum_out, uint32_t mf_in,
                   uint32_t mf_out, hipStream_t st) {
        hipLaunchKernelGGL((k_reduce_requant<BITS, LPG, SR>), dim3(grid_for(n_lanes)), dim3(kBlock), 0, st, peers, n_peers,
                           n_lanes, out, sum_out, mf_in, mf_out);
        return launch_status();
    }
};
template <int BITS, int LPG, bool SR> struct LaunchDispatch {
    static int run(const void* x, uint64_t n_lanes, uint32_t lanes_per_row, uint32_t K, const int32_t* dest, uint8_t* send,
                   const RowLayout& rl, uint32_t meta_fp32, hipStream_t st) {
        hipLaunchKernelGGL((k_dispatch_quant<BITS, LPG, SR>), dim3(grid_for(n_lanes)), dim3(kBlock), 0, st, (const uint4*)x,
                           n_lanes, lanes_per_row, K, dest, send, rl, meta_fp32);
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
    const uint64_t meta = (fmt->flags & FCV2_F_META_FP32) ? 4 : 2;
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

int fcv2_quantize_pack(const void* x, uint64_t n, const fcv2_fmt_t* fmt, void* packed, void* stream) {
    if (!x || !packed || !fmt) return FCV2_ERR_INVALID_ARG;
    fcv2_layout_t l;
    int rc = fcv2_get_layout(n, fmt, FCV2_TENSOR_ALIGN, &l);
    if (rc != FCV2_OK) return rc;
    if (!aligned16(x) || !aligned16(packed)) return FCV2_ERR_ALIGN;
    return by_format<LaunchQuantize>(fmt, x, n / 8, sections_of(packed, l), (uint32_t)((fmt->flags & FCV2_F_META_FP32) != 0),
                                     (hipStream_t)stream);
}

int fcv2_unpack_dequant(const void* packed, uint64_t n, const fcv2_fmt_t* fmt, void* out, int out_dtype, void* stream) {
    if (!packed || !out || !fmt) return FCV2_ERR_INVALID_ARG;
    if (out_dtype != FCV2_DT_BF16 && out_dtype != FCV2_DT_FP32) return FCV2_ERR_INVALID_ARG;
    fcv2_layout_t l;
    int rc = fcv2_get_layout(n, fmt, FCV2_TENSOR_ALIGN, &l);
    if (rc != FCV2_OK) return rc;
    if (!aligned16(packed) || !aligned16(out)) return FCV2_ERR_ALIGN;
    return by_format<LaunchUnpack>(fmt, sections_of(packed, l), n / 8, out, (uint32_t)(out_dtype == FCV2_DT_FP32),
                                   (uint32_t)((fmt->flags & FCV2_F_META_FP32) != 0), (hipStream_t)stream);
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
    if (fmt_in->bits != fmt_out->bits || fmt_in->group != fmt_out->group ||
        ((fmt_in->flags ^ fmt_out->flags) & FCV2_F_SPIKE) != 0)
        return FCV2_ERR_UNSUPPORTED;
    if (!aligned16(packed_out) || (sum_out && !aligned16(sum_out))) return FCV2_ERR_ALIGN;
    PeerArgs pa;
    for (int p = 0; p < FCV2_MAX_PEERS; ++p) {
        const void* ptr = peers[p < n_peers ? p : 0];
        if (!ptr) return FCV2_ERR_INVALID_ARG;
        if (!aligned16(ptr)) return FCV2_ERR_ALIGN;
        pa.s[p] = sections_of(ptr, lin);
    }
    return by_format<LaunchReduce>(fmt_in, pa, n_peers, n / 8, sections_of(packed_out, lout), sum_out,
                                   (uint32_t)((fmt_in->flags & FCV2_F_META_FP32) != 0),
                                   (uint32_t)((fmt_out->flags & FCV2_F_META_FP32) != 0), (hipStream_t)stream);
}

int fcv2_dispatch_workspace_bytes(uint32_t T, uint32_t K, uint32_t E, size_t* out) {
    if (!out || T == 0 || K == 0 || E == 0) return FCV2_ERR_INVALID_ARG;
    if ((uint64_t)T * K > 0x7FFFFFFFull) return FCV2_ERR_INVALID_ARG;
    if (E > 8192) return FCV2_ERR_UNSUPPORTED;  // per-wave expert counters live in LDS
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
    hipLaunchKernelGGL(k_dispatch_scan_experts, dim3(1), dim3(256), 0, st, totals, E, expert_offsets);
    hipLaunchKernelGGL(k_dispatch_rank, dim3(w.n_chunks), dim3(kChunk), (kChunk / 64) * E * 4, st, ids, w.n_slots, E, hist,
                       expert_offsets, dest, row_src);
    if (launch_status() != FCV2_OK) return FCV2_ERR_LAUNCH;
    RowLayout rl;
    auto rel = [](uint64_t o) { return o == FCV2_ABSENT ? 0u : (uint32_t)o; };
    rl.plane8 = rel(l.off_plane8);
    rl.plane4 = rel(l.off_plane4);
    rl.plane2 = rel(l.off_plane2);
    rl.plane1 = rel(l.off_plane1);
    rl.scale = rel(l.off_scale);
    rl.zero = rel(l.off_zero);
    rl.spike_val = rel(l.off_spike_val);
    rl.spike_idx = rel(l.off_spike_idx);
    rl.row_bytes = (uint32_t)l.total_bytes;
    return by_format<LaunchDispatch>(fmt, x, (uint64_t)T * H / 8, H / 8, K, (const int32_t*)dest, (uint8_t*)send, rl,
                                     (uint32_t)((fmt->flags & FCV2_F_META_FP32) != 0), st);
}

}  // extern "C"
