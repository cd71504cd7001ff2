// fcv2_quantize.hip -- fcv2_quantize_pack(_slices): the sender-side kernel and its launch.
#include "fcv2_host.h"

namespace fcv2 {

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
    // refill of a set is issued right after the tile that used it has been stored.  Loads are unconditional:
    // conditional ones would force full waits.  A refill past the wave's last tile asks for one 16-byte piece of the
    // tensor's last tile in every lane (a single cache line per load instead of sixteen) and is never used.
    const uint32_t last = n_tiles - 1;
    auto fetch = [&](uint32_t t) {
        const bool real = t < n_tiles;
        const uint32_t tt = real ? t : last;
        return tile_load(x, (uint64_t)tt * 256, lane, real ? n_pieces - tt * 256 : 1u);
    };
    TileIn a = fetch(tile);
    TileIn b = fetch(tile + stride);
    while (true) {
        process(a, tile);
        a = fetch(tile + 2 * stride);
        tile += stride;
        if (tile >= n_tiles) break;
        process(b, tile);
        b = fetch(tile + 2 * stride);
        tile += stride;
        if (tile >= n_tiles) break;
    }
}

// Launch shape.  A compute unit holds 8 blocks of the quantize kernel (64 registers per lane, 22 KiB of LDS per block).
// A tensor of at most that many tiles gets one wave per tile; a larger one gets 4 blocks per compute unit, each wave
// walking several tiles with the next loads in flight.  In the first case the waves of a launch form a single
// generation (all load, then all compute, then all store); from 4 bits up, where a record is a larger part of the
// traffic, it measured 2 to 6 % faster on the 16 M-element tensor to let only 4 blocks into a compute unit at a time, so
// that the later blocks' loads run under the earlier blocks' stores (3 and 5 to 7 blocks: slower; at 2 and 3 bits all 8
// are faster).  The limit is set with unused dynamic LDS.  The compute-unit count is asked of the current device at
// every call (a cheap attribute read): nothing is cached, so a process that moves between devices, or calls from
// several threads, always gets the count of the device it launches on.
struct QuantizeLaunch {
    unsigned blocks;
    size_t lds_pad;
};
static QuantizeLaunch quantize_launch_shape(uint32_t n_tiles, int bits) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        cus = 256;
    const unsigned need = (n_tiles + kWaves - 1) / kWaves;
    const bool one_tile_per_wave = need <= 8u * (unsigned)cus;
    const unsigned blocks = (one_tile_per_wave ? 8u : 4u) * (unsigned)cus;
    QuantizeLaunch q;
    q.blocks = need < blocks ? need : blocks;
    // 160 KiB of LDS per compute unit: blocks of 36 KiB fit four times, not five, whatever the allocation granule
    constexpr size_t kStatic = sizeof(uint4) * kWaves * 64 * kRowU4 + sizeof(float) * kScaleTables;
    q.lds_pad = (one_tile_per_wave && bits >= 4 && need > 4u * (unsigned)cus) ? (size_t)36864 - kStatic : 0;
    return q;
}

template <int BITS, int G, bool SR> struct LaunchQuantize {
    static int run(const void* x, uint64_t n, void* out, const Rec& rec, uint32_t meta_mode, uint32_t n_slices,
                   uint64_t record_stride, hipStream_t st) {
        constexpr int EPL = kEplStream;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        const uint32_t n_tiles = (n_lanes + 63) / 64;
        const QuantizeLaunch q = quantize_launch_shape(n_tiles, BITS);
        if (meta_mode == kMetaInt)
            return launch(k_quantize_pack_t<BITS, G / EPL, SR, true>, dim3(q.blocks), dim3(kBlock), q.lds_pad, st,
                          (const uint4*)x, n_lanes, (uint8_t*)out, rec, meta_mode, n_lanes / n_slices, record_stride);
        return launch(k_quantize_pack_t<BITS, G / EPL, SR, false>, dim3(q.blocks), dim3(kBlock), q.lds_pad, st,
                      (const uint4*)x, n_lanes, (uint8_t*)out, rec, meta_mode, n_lanes / n_slices, record_stride);
    }
};
int launch_quantize(const fcv2_fmt_t* fmt, const void* x, uint64_t n, void* out, const Rec& rec, uint32_t n_slices,
                    uint64_t record_stride, hipStream_t st) {
    return by_format<LaunchQuantize>(fmt, x, n, out, rec, meta_mode_of(fmt), n_slices, record_stride, st);
}

}  // namespace fcv2
