// fcv2_reduce.hip -- fcv2_reduce_requant: the local step of the two-step AllReduce (Sections 3.1, 3.4), kernels and launch.
#include "fcv2_host.h"

namespace fcv2 {

// Local reduce step.  EPL = 16 elements per lane (groups of 32 are two lanes, larger ones four to sixteen).
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
    const uint32_t L = xcd_tile_block(blockIdx.x, gridDim.x) * kBlock + threadIdx.x;
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
        auto add_peer = [&](const RawPlanes<EPL>& r, uint32_t mraw, uint32_t mraw2) {
            const GroupMeta m = spread_meta<LPG, SR, INT_META>(mraw, mraw2, mo, tabs);
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
            uint32_t mraw[CH], mraw2[CH];
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const BufferSrc src = buffer_src(peers.base[p + i], rec_in.total);
                r[i] = load_planes<BITS, EPL>(src, rec_in, L);
                mraw[i] = ld32(src, mo.at);
                mraw2[i] = (LPG < 4 && SR) ? ld32(src, mo.at2) : 0u;
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) add_peer(r[i], mraw[i], mraw2[i]);
        }
        for (; p < n_peers; ++p) {
            const BufferSrc src = buffer_src(peers.base[p], rec_in.total);
            const RawPlanes<EPL> r = load_planes<BITS, EPL>(src, rec_in, L);
            const uint32_t mraw = ld32(src, mo.at);
            const uint32_t mraw2 = (LPG < 4 && SR) ? ld32(src, mo.at2) : 0u;
            add_peer(r, mraw, mraw2);
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
    const uint32_t L = xcd_tile_block(blockIdx.x, gridDim.x) * kBlock + threadIdx.x;
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
        const uint32_t mraw2 = (LPG < 4 && SR) ? ld32(src, mo.at2) : 0u;
        const GroupMeta m = (meta_mode_in == kMetaInt) ? spread_meta<LPG, SR, true>(mraw, mraw2, mo, tabs)
                                                       : spread_meta<LPG, SR, false>(mraw, mraw2, mo, tabs);
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

template <int BITS, int G, bool SR> struct LaunchReduce {
    static int run(const PeerPtrs& peers, int n_peers, uint64_t n, const Rec& rec_in, void* out, const Rec& rec_out,
                   float* sum_out, uint32_t mf_in, uint32_t mf_out, hipStream_t st) {
        constexpr int EPL = 16;  // 32 was measured: 180 VGPRs, two waves per SIMD, 15 % slower; 8 doubles the per-lane work
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        return launch(k_reduce_requant<BITS, EPL, G / EPL, SR>, dim3(grid_lanes_xcd(n_lanes)), dim3(kBlock), 0, st, peers, n_peers,
                      n_lanes, rec_in, (uint8_t*)out, rec_out, sum_out, mf_in, mf_out);
    }
};
template <int BITS, int G, bool SR> struct LaunchReduceMixed {  // BITS = output width
    static int run(const PeerPtrs& peers, int n_peers, uint32_t bits_in, uint64_t n, const Rec& rec_in, void* out,
                   const Rec& rec_out, float* sum_out, uint32_t mf_in, uint32_t mf_out, hipStream_t st) {
        constexpr int EPL = 16;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        return launch(k_reduce_requant_mixed<BITS, EPL, G / EPL, SR>, dim3(grid_lanes_xcd(n_lanes)), dim3(kBlock), 0, st, peers,
                      n_peers, bits_in, n_lanes, rec_in, (uint8_t*)out, rec_out, sum_out, mf_in, mf_out);
    }
};
int launch_reduce(const fcv2_fmt_t* fmt_in, const fcv2_fmt_t* fmt_out, const PeerPtrs& peers, int n_peers, uint64_t n,
                  const Rec& rec_in, void* out, const Rec& rec_out, float* sum_out, hipStream_t st) {
    const uint32_t mf_in = meta_mode_of(fmt_in), mf_out = meta_mode_of(fmt_out);
    if (fmt_in->bits != fmt_out->bits)
        return by_format<LaunchReduceMixed>(fmt_out, peers, n_peers, fmt_in->bits, n, rec_in, out, rec_out, sum_out, mf_in, mf_out, st);
    return by_format<LaunchReduce>(fmt_in, peers, n_peers, n, rec_in, out, rec_out, sum_out, mf_in, mf_out, st);
}

}  // namespace fcv2
