// fcv2_reduce.hip -- fcv2_reduce_requant: the local step of the two-step AllReduce (Sections 3.1, 3.4), kernels and launch.
#include "fcv2_host.h"

// Elements per lane, waves per SIMD, peers in flight and the way spikes are restored, with what was measured on the
// MI355X (16 M-element payload, 8 peers, inputs not in the last-level cache, us per launch, runs on one machine):
//   at 2 / 3 / 4 / 5 / 6 / 7 / 8 bits, 16 elements per lane: overlay at 2 and 3 bits and park above (the choice below)
//   26.2 / 28.3 / 27.7 / 32.2 / 32.5 / 38.3 / 34.1; park everywhere 26.6 / 28.2 / 27.7 / 32.3 / 32.4 / 38.2 / 34.1;
//   32 elements per lane (112 registers, four waves per SIMD; five spill): within 1 us of 16 at every width, not better;
//   one peer in flight at eight waves 29.7 at 3 bits, two at seven waves 28.5, the next two peers requested under the
//   decoding of the current two 29.6 (against 28.8 in that run).
// The peer loop costs the same per element either way (the FMA, the add and the unpacking are per element); what 32
// elements per lane save in per-lane work they lose in occupancy.
#ifndef FCV2_REDUCE_EPL
#define FCV2_REDUCE_EPL(G) 16
#endif
#ifndef FCV2_REDUCE_WAVES32
#define FCV2_REDUCE_WAVES32 4
#endif
#ifndef FCV2_REDUCE_WAVES16
#define FCV2_REDUCE_WAVES16 6
#endif
#ifndef FCV2_REDUCE_CH
#define FCV2_REDUCE_CH 2
#endif
#ifndef FCV2_REDUCE_PATCH
#define FCV2_REDUCE_PATCH(BITS) ((BITS) <= 3 ? kPatchOverlay : kPatchPark)
#endif

namespace fcv2 {

// Local reduce step.  EPL = 16 elements per lane (groups of 32 are two lanes, larger ones four to sixteen).
//  - codes are unpacked into 16-bit halves and fed to v_fma_mix_f32 as fp16 denormals (q * 2^-24) against the
//    scale pre-multiplied by 2^24: the product is the same real number q * scale, the FMA rounds once, so the
//    result is bit-identical to fma(float(q), scale, lo) without a conversion instruction per element;
//  - the spikes of every peer are put back through a private row in LDS: a dynamic register index done by memory.
// Spike restoration (Section 3.3: after dequantization the two spikes of a group go back to their places).  A spike
// position is a dynamic index into the lane's registers, which only memory can do; each lane has a private row of 16
// dwords in LDS for it, and a lane's EPL elements are handled 16 at a time.  Two ways, chosen per bit width:
//   park:    a lane that owns a spike in these 16 elements writes its 16 decoded values to the row, overwrites the
//            spike slot and reads the row back.  No extra arithmetic, 8 sixteen-byte LDS operations.
//   overlay: the row is all zero between uses.  The wire format stores code 0 at a spike position, so what the decoder
//            puts there is t = fma(0, scale, zero), the same for the whole group and known without looking: the owner
//            writes (spike bits XOR t bits) into the slot, every lane reads its row back and XORs it onto its decoded
//            values on their way into the accumulators (t ^ spike ^ t = spike, everything else ^ 0 stays), the owner
//            puts the zero back.  Half the LDS traffic, one cheap XOR per element.  Records whose code at a spike
//            position is not 0 are malformed; with the overlay their spikes come back wrong.
// LDS is shared by the four SIMDs of a compute unit and the park's traffic alone fills most of it at the low widths,
// while the overlay's XORs land on the VALUs, which are the other thing this kernel runs out of.
constexpr int kPatchPark = 0, kPatchOverlay = 1;

// Which register of Q[8], and which half of it, holds element e of 16; by how much its code is shifted inside the half.
template <int BITS> struct UnitPairMap {  // codes_pairs on two units of 8: unit u = Q[4u..4u+3], element k and k + 4, at bit 0
    static constexpr int k_of(int e) { return 4 * (e >> 3) + (e & 3); }
    static constexpr bool in_hi(int e) { return ((e >> 2) & 1) != 0; }
    static constexpr int pos(int) { return 0; }
};

// (Measured and not used: taking the spread of the 3-bit format's extra bits from two 256-entry LDS tables instead of
// computing it -- 12 VALU cycles instead of 35 per peer and 16 elements -- made the kernel 7 % slower: two more LDS
// reads at scattered addresses per peer, in front of everything else the peer needs.)
template <int BITS, int EPL, bool SR, int PATCH>
__device__ __forceinline__ void add_peer_values(const RawPlanes<EPL>& r, const GroupMeta& m, uint32_t lig, uint4* row, float (&acc)[EPL]) {
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    using P = Planes<BITS>;
    constexpr bool IN_PLACE = BITS <= 4;  // narrow codes are only masked where they stand (codes_pairs16)
    using M = typename std::conditional<IN_PLACE, PairMap<(IN_PLACE ? BITS : 2)>, UnitPairMap<BITS>>::type;
    const float s = m.s, lo = m.lo;
    uint32_t relmin = 0xFFFFFFFFu, relmax = 0xFFFFFFFFu, t = 0u;
    if (SR) {
        relmin = (m.si & 0xFFu) - lig * (uint32_t)EPL;  // position inside this lane, or >= EPL when another lane owns the spike
        relmax = (m.si >> 8) - lig * (uint32_t)EPL;
        if (PATCH == kPatchOverlay) t = f2u(__fmaf_rn(0.0f, s, lo));  // what a zero code decodes to (-0 offsets, infinite scales included)
    }
    const uint32_t smin = m.sv << 16, smax = m.sv & 0xFFFF0000u;
    u32a* o = reinterpret_cast<u32a*>(row);
    float mult[9];
#pragma unroll
    for (int q = 0; q < 9; ++q) mult[q] = s * __builtin_ldexpf(1.0f, 24 - q);  // only the positions in use survive
    // Decoding exists twice: for scales below 2^100 (always, unless the data spans more than that: 2^24 * scale could
    // overflow) codes go into the mixed-precision FMA as fp16 denormals; otherwise they are converted one by one.
    // codes16 prepares the 16 codes of half h in the form its kind of decoding takes, value decodes element e of them.
    struct Codes16 {
        uint32_t Q[8];
        float qf[16];
    };
    auto codes16 = [&](auto fast_tag, int h, Codes16& c) {
        if constexpr (decltype(fast_tag)::value) {
            if constexpr (IN_PLACE) {
                const uint32_t p1 = P::w1 ? (EPL == 16 ? r.p1 : (h == 0 ? and_lit<0xFFFFu>(r.p1) : r.p1 >> 16)) : 0u;
                codes_pairs16<BITS>(P::w4 ? r.p4[(2 * h) % (EPL / 8)] : 0u, P::w4 ? r.p4[(2 * h + 1) % (EPL / 8)] : 0u,
                                    P::w2 ? r.p2[h % ((EPL + 15) / 16)] : 0u, p1, c.Q);
            } else {
#pragma unroll
                for (int uu = 0; uu < 2; ++uu) {
                    const int u = 2 * h + uu;
                    uint32_t Q4[4];
                    const uint32_t p4 = P::w4 ? r.p4[u] : 0u;
                    const uint32_t p2 = P::w2 ? ((r.p2[u >> 1] >> (16 * (u & 1))) & 0xFFFFu) : 0u;
                    const uint32_t p1 = P::w1 ? ((r.p1 >> (8 * u)) & 0xFFu) : 0u;
                    codes_pairs<BITS>(P::w8 ? r.p8[2 * u] : 0u, P::w8 ? r.p8[2 * u + 1] : 0u, p4, p2, p1, Q4);
#pragma unroll
                    for (int k = 0; k < 4; ++k) c.Q[4 * uu + k] = Q4[k];
                }
            }
        } else {
#pragma unroll
            for (int uu = 0; uu < 2; ++uu) {
                float q8[8];
                unit_codes<BITS, EPL>(r, 2 * h + uu, q8);
#pragma unroll
                for (int j = 0; j < 8; ++j) c.qf[8 * uu + j] = q8[j];
            }
        }
    };
    auto value = [&](auto fast_tag, const Codes16& c, int e) -> float {
        if constexpr (!decltype(fast_tag)::value) {
            return __fmaf_rn(c.qf[e], s, lo);
        } else {
            const half2v hh = __builtin_bit_cast(half2v, c.Q[M::k_of(e)]);
            return __builtin_fmaf(M::in_hi(e) ? (float)hh.y : (float)hh.x, mult[M::pos(M::k_of(e))], lo);
        }
    };
    if constexpr (SR && PATCH == kPatchOverlay) {
        // everything of a peer inside one branch on the scale: the decoded values go straight into the accumulators, a
        // quarter at a time, so that they are never all live at once
        auto body = [&](auto fast_tag) {
#pragma unroll
            for (int h = 0; h < EPL / 16; ++h) {
                const uint32_t rmin = relmin - 16u * h, rmax = relmax - 16u * h;  // the same inside these 16 elements
                if (rmin < 16u) o[rmin] = smin ^ t;
                if (rmax < 16u) o[rmax] = smax ^ t;
                Codes16 c;
                codes16(fast_tag, h, c);
#pragma unroll
                for (int i = 0; i < 4; ++i) {  // a wave's LDS operations execute in issue order: these reads see the writes above
                    const uint4 x4 = row[i];
                    const uint32_t x[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int e = 4 * i + b;
                        acc[16 * h + e] = __fadd_rn(acc[16 * h + e], u2f(f2u(value(fast_tag, c, e)) ^ x[b]));
                    }
                }
                if (rmin < 16u) o[rmin] = 0u;  // ... and these zeros land after them
                if (rmax < 16u) o[rmax] = 0u;
            }
        };
        if (s < 0x1p+100f)
            body(std::true_type{});
        else
            body(std::false_type{});
    } else {
        // only the decoding sits inside the branch on the scale; parking and accumulating follow it once
#pragma unroll
        for (int h = 0; h < EPL / 16; ++h) {
            float v[16];
            if (s < 0x1p+100f) {
                Codes16 c;
                codes16(std::true_type{}, h, c);
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = value(std::true_type{}, c, e);
            } else {
                Codes16 c;
                codes16(std::false_type{}, h, c);
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = value(std::false_type{}, c, e);
            }
            if (SR) {
                const uint32_t rmin = relmin - 16u * h, rmax = relmax - 16u * h;
                if (rmin < 16u || rmax < 16u) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) row[i] = make_uint4(f2u(v[4 * i]), f2u(v[4 * i + 1]), f2u(v[4 * i + 2]), f2u(v[4 * i + 3]));
                    if (rmin < 16u) o[rmin] = smin;
                    if (rmax < 16u) o[rmax] = smax;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint4 a = row[i];
                        v[4 * i] = u2f(a.x);
                        v[4 * i + 1] = u2f(a.y);
                        v[4 * i + 2] = u2f(a.z);
                        v[4 * i + 3] = u2f(a.w);
                    }
                }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[16 * h + e] = __fadd_rn(acc[16 * h + e], v[e]);
        }
    }
}

template <int BITS, int EPL, int LPG, bool SR, int PATCH>
// Peers are taken two at a time (both peers' loads issued before either is decoded).  Every peer in flight costs
// about 15 registers; with two the kernel needs 65 to 74 and six or seven waves fit a SIMD, which measured faster
// than four peers in flight at four or five waves, and faster than one peer at eight.
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(EPL == 32 ? FCV2_REDUCE_WAVES32 : FCV2_REDUCE_WAVES16)))
void k_reduce_requant(PeerPtrs peers, int n_peers, uint32_t n_lanes, Rec rec_in,
                                                           uint8_t* __restrict__ out, Rec rec_out, float* __restrict__ sum_out,
                                                           uint32_t meta_mode_in, uint32_t meta_mode_out) {
    constexpr int CH = FCV2_REDUCE_CH;  // peers in flight
    constexpr int ROW = 16 / 4 + 1;  // uint4 per private row of 16 dwords, one of padding: conflict-free 16-byte accesses
    __shared__ uint4 lds[kBlock * ROW];  // 20 KiB: eight blocks fill the 160 KiB of a compute unit exactly
    extern __shared__ float tabs[];      // the scale tables of the integer metadata: dynamic, present only when a format uses them
    if (meta_mode_in == kMetaInt || meta_mode_out == kMetaInt) fill_scale_tables(tabs);
    const uint32_t L = xcd_tile_block(blockIdx.x, gridDim.x) * kBlock + threadIdx.x;
    if (L >= n_lanes) return;
    const uint32_t lig = threadIdx.x & (LPG - 1);
    uint4* row = &lds[threadIdx.x * ROW];
    if (SR && PATCH == kPatchOverlay) {  // the lane's overlay row starts, and is left after every use, all zero
#pragma unroll
        for (int i = 0; i < 4; ++i) row[i] = make_uint4(0u, 0u, 0u, 0u);
    }
    const MetaOffsets mo = meta_offsets<LPG, SR>(rec_in, L, meta_mode_in);
    // -0 is the identity of fp32 addition for every value including -0, so the chain below starts exactly at v_0
    float acc[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) acc[j] = -0.0f;
    // The peer loop exists twice, once per kind of metadata decoding, chosen by one uniform branch outside it.
    auto sum_peers = [&](auto int_meta) {
        constexpr bool INT_META = decltype(int_meta)::value;
        auto add_peer = [&](const RawPlanes<EPL>& r, uint32_t mraw, uint32_t mraw2) {
            const GroupMeta m = spread_meta<LPG, SR, INT_META>(mraw, mraw2, mo, tabs, rec_in.idx_bf16);
            add_peer_values<BITS, EPL, SR, PATCH>(r, m, lig, row, acc);
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
// (one uniform switch around the peer loop), the output width stays a template parameter.  A compatibility path next to
// the specialised kernel above: spikes always through the park, no choice of occupancy per width.
template <int BITS_OUT, int EPL, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_reduce_requant_mixed(PeerPtrs peers, int n_peers, uint32_t bits_in, uint32_t n_lanes,
                                                                 Rec rec_in, uint8_t* __restrict__ out, Rec rec_out,
                                                                 float* __restrict__ sum_out, uint32_t meta_mode_in,
                                                                 uint32_t meta_mode_out) {
    constexpr int ROW = 16 / 4 + 1;
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
    // One uniform switch on the input width around the whole peer loop; inside it peers are taken two at a time, both
    // peers' loads issued before either is decoded (an odd last peer is requested twice and added once).
    auto sum_peers = [&](auto bits_tag) {
        constexpr int B = decltype(bits_tag)::value;
        auto add_peer = [&](const RawPlanes<EPL>& r, uint32_t mraw, uint32_t mraw2) {
            const GroupMeta m = (meta_mode_in == kMetaInt) ? spread_meta<LPG, SR, true>(mraw, mraw2, mo, tabs, rec_in.idx_bf16)
                                                           : spread_meta<LPG, SR, false>(mraw, mraw2, mo, tabs, rec_in.idx_bf16);
            add_peer_values<B, EPL, SR, kPatchPark>(r, m, lig, row, acc);
        };
        for (int p = 0; p < n_peers; p += 2) {
            const bool two = p + 1 < n_peers;
            RawPlanes<EPL> r[2];
            uint32_t mraw[2], mraw2[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const BufferSrc src = buffer_src(peers.base[(i == 1 && two) ? p + 1 : p], rec_in.total);
                r[i] = load_planes<B, EPL>(src, rec_in, L);
                mraw[i] = ld32(src, mo.at);
                mraw2[i] = (LPG < 4 && SR) ? ld32(src, mo.at2) : 0u;
            }
            add_peer(r[0], mraw[0], mraw2[0]);
            if (two) add_peer(r[1], mraw[1], mraw2[1]);
        }
    };
    switch (bits_in) {
        case 2: sum_peers(std::integral_constant<int, 2>{}); break;
        case 3: sum_peers(std::integral_constant<int, 3>{}); break;
        case 4: sum_peers(std::integral_constant<int, 4>{}); break;
        case 5: sum_peers(std::integral_constant<int, 5>{}); break;
        case 6: sum_peers(std::integral_constant<int, 6>{}); break;
        case 7: sum_peers(std::integral_constant<int, 7>{}); break;
        default: sum_peers(std::integral_constant<int, 8>{}); break;
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
        constexpr int EPL = FCV2_REDUCE_EPL(G);
        constexpr int PATCH = FCV2_REDUCE_PATCH(BITS);
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        const size_t tab_bytes = (mf_in == kMetaInt || mf_out == kMetaInt) ? sizeof(float) * kScaleTables : 0;
        return launch(k_reduce_requant<BITS, EPL, G / EPL, SR, PATCH>, dim3(grid_lanes_xcd(n_lanes)), dim3(kBlock), tab_bytes, st, peers,
                      n_peers, n_lanes, rec_in, (uint8_t*)out, rec_out, sum_out, mf_in, mf_out);
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
