// fcv2_quantize.hip -- fcv2_quantize_pack(_slices): the sender-side kernel and its launch.
#include "fcv2_host.h"

namespace fcv2 {

// Sender: one wave per tile of 64 x 32 elements.  (Persistent waves that walk several tiles with the next tile's loads in
// flight measured 4 to 15 % slower on tensors of 32 M and 64 M elements: with far more waves than the chip holds, the
// hardware's own succession of blocks overlaps one block's stores with the next block's loads better.)
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
    const uint32_t tile = blockIdx.x * kWaves + wave;
    if (tile >= n_tiles) return;
    // pieces past the end of the tensor re-read the last valid one (tile_load): the lanes that own them store nothing
    const TileIn t = tile_load(x, (uint64_t)tile * 256, lane, n_lanes * 4 - tile * 256);
    uint32_t w[16];
    tile_transpose(t, lds[wave], lane, w);
    const uint32_t slice = (tile * 64) / slice_lanes;  // uniform
    const uint32_t L = tile * 64 + lane;
    if (L < n_lanes) {  // groups never straddle the end: whole groups are in or out together
        uint32_t c[EPL / 4];
        GroupMeta m;
        quantize_lane<BITS, EPL, LPG, SR>(w, lig, meta_mode, tabs, &lds[wave][lane * kRowU4], c, m);
        uint8_t* o = out + slice * record_stride;
        const uint32_t Lr = L - slice * slice_lanes;  // lane inside the record
        store_planes<BITS, EPL>(o, rec, Lr, c);
        if (lig == 0) store_meta<SR>(o, rec, Lr / LPG, m, meta_mode);
    }
}

// Launch shape: one block per four tiles.  A compute unit holds 8 blocks of the kernel (32 to 65 registers per lane, 16 to
// 18 KiB of LDS per block), and at 2 to 7 bits that is the fastest at every size measured (16 M, 32 M, 64 M elements).  At 8 bits,
// where the record is a third of the traffic, tensors of more blocks than the chip holds at once ran 6 % (32 M) and
// 10 % (64 M) faster with only 4 blocks in a compute unit at a time: later blocks' loads then run under earlier blocks'
// stores.  The limit is set with unused dynamic LDS.  The compute-unit count is asked of the current device at every call
// (a cheap attribute read): nothing is cached, so a process that moves between devices, or calls from several threads,
// always gets the count of the device it launches on.
struct QuantizeLaunch {
    unsigned blocks;
    size_t lds_pad;
};
static QuantizeLaunch quantize_launch_shape(uint32_t n_tiles, int bits) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        cus = 256;
    QuantizeLaunch q;
    q.blocks = (n_tiles + kWaves - 1) / kWaves;
    // 160 KiB of LDS per compute unit: blocks of 36 KiB fit four times, not five, whatever the allocation granule
    constexpr size_t kStatic = sizeof(uint4) * kWaves * 64 * kRowU4 + sizeof(float) * kScaleTables;
    q.lds_pad = (bits == 8 && q.blocks > 8u * (unsigned)cus) ? (size_t)36864 - kStatic : 0;
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
