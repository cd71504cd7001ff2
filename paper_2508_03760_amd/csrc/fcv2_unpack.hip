// fcv2_unpack.hip -- fcv2_unpack_dequant(_slices): the receiver-side kernel and its launch.
#include "fcv2_host.h"

namespace fcv2 {

// Receiver: 32 elements per lane; every lane reads its group's metadata itself.  The results go through LDS so that
// (a) the two spikes of a group are dropped into place by plain indexed LDS writes of the lanes that own their
// positions (Section 3.3: restored in place) and (b) the global stores are fully coalesced 16-byte pieces.
template <int BITS, int LPG, bool SR, bool OUT_FP32>
__global__ __launch_bounds__(kBlock) void k_unpack_dequant_t(PeerPtrs records, uint32_t slice_lanes, Rec rec, uint32_t n_lanes,
                                                             uint4* __restrict__ out, uint32_t meta_mode) {
    constexpr int EPL = kEplStream;
    constexpr int ROW = OUT_FP32 ? 9 : 5;  // uint4 per lane row incl. one of padding
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
            si = rec.idx_bf16 ? idx_pair_of_bf16(*reinterpret_cast<const uint32_t*>(in + (rec.spike_idx + 4u * g)))
                              : (uint32_t) * reinterpret_cast<const uint16_t*>(in + (rec.spike_idx + 2u * g));
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
        if (piece0 + P < n_pieces) store_stream(&out[(uint64_t)piece0 + P], lds[wave][(P / NP) * ROW + (P % NP)]);
    }
}

template <int BITS, int G, bool SR> struct LaunchUnpack {
    static int run(const PeerPtrs& records, uint32_t n_slices, const Rec& rec, uint64_t n, void* out, uint32_t out_fp32,
                   uint32_t meta_mode, hipStream_t st) {
        constexpr int EPL = kEplStream;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        if (out_fp32)
            return launch(k_unpack_dequant_t<BITS, G / EPL, SR, true>, dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st, records,
                          n_lanes / n_slices, rec, n_lanes, (uint4*)out, meta_mode);
        return launch(k_unpack_dequant_t<BITS, G / EPL, SR, false>, dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st, records,
                      n_lanes / n_slices, rec, n_lanes, (uint4*)out, meta_mode);
    }
};
int launch_unpack(const fcv2_fmt_t* fmt, const PeerPtrs& records, uint32_t n_slices, const Rec& rec, uint64_t n, void* out,
                  uint32_t out_fp32, hipStream_t st) {
    return by_format<LaunchUnpack>(fmt, records, n_slices, rec, n, out, out_fp32, meta_mode_of(fmt), st);
}

}  // namespace fcv2
