// fcv2_host.h -- host-side glue shared by the translation units of libfcv2: format dispatch, launch helpers, and
// the per-call launch functions each kernel file exports to the C ABI in fcv2_api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "fcv2_device.h"

namespace fcv2 {

static inline uint32_t meta_mode_of(const fcv2_fmt_t* f) {
    return (f->flags & FCV2_F_META_INT) ? kMetaInt : (f->flags & FCV2_F_META_FP32) ? kMetaFp32 : kMetaBf16;
}

static inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

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

// Enqueues `kernel` and returns the status of THIS launch.  The arguments are converted to the kernel's own parameter
// types and handed to hipLaunchKernel, whose return value is the launch's own: the runtime's "last error" slot, which
// other code of the process may have set and may still want to read, is neither consulted nor cleared.
template <typename... KArgs, typename... Args>
static inline int launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st, Args&&... args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count differs from the kernel's parameter count");
    std::tuple<KArgs...> vals{static_cast<KArgs>(std::forward<Args>(args))...};
    void* ptrs[sizeof...(KArgs)];
    std::apply([&](auto&... v) { size_t i = 0; ((ptrs[i++] = (void*)&v), ...); }, vals);
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, st) == hipSuccess ? FCV2_OK
                                                                                                                   : FCV2_ERR_LAUNCH;
}

static inline unsigned grid_lanes(uint32_t n_lanes) { return (unsigned)((n_lanes + kBlock - 1) / kBlock); }
// the same padded to a multiple of the 8 XCDs, for kernels that map block ids with xcd_tile_block
static inline unsigned grid_lanes_xcd(uint32_t n_lanes) { return (grid_lanes(n_lanes) + 7u) & ~7u; }

constexpr int kChunk = 256;  // routed slots per block in the dispatch planning kernels

struct DispatchWs {  // carving of the dispatch workspace
    uint32_t n_slots, n_chunks;
    size_t off_hist, off_totals, off_lrank, off_dest, bytes;
};
static DispatchWs dispatch_ws(uint32_t T, uint32_t K, uint32_t E) {
    DispatchWs w;
    w.n_slots = T * K;
    w.n_chunks = (w.n_slots + kChunk - 1) / kChunk;
    w.off_hist = 0;                                                                 // [n_chunks][E] int32
    w.off_totals = round_up((size_t)w.n_chunks * E * 4, 256);                        // [E] int32
    w.off_lrank = w.off_totals + round_up((size_t)E * 4, 256);                       // [n_slots] bytes: rank inside the chunk
    w.off_dest = w.off_lrank + round_up((size_t)w.n_slots, 256);                     // [n_slots] int32: only the direct kernel reads it
    w.bytes = w.off_dest + round_up((size_t)w.n_slots * 4, 256);
    return w;
}

// One function per call, defined next to its kernels.  Arguments are checked by the C ABI functions before.
int launch_quantize(const fcv2_fmt_t* fmt, const void* x, uint64_t n, void* out, const Rec& rec, uint32_t n_slices,
                    uint64_t record_stride, hipStream_t st);
int launch_unpack(const fcv2_fmt_t* fmt, const PeerPtrs& records, uint32_t n_slices, const Rec& rec, uint64_t n, void* out,
                  uint32_t out_fp32, hipStream_t st);
int launch_reduce(const fcv2_fmt_t* fmt_in, const fcv2_fmt_t* fmt_out, const PeerPtrs& peers, int n_peers, uint64_t n,
                  const Rec& rec_in, void* out, const Rec& rec_out, float* sum_out, hipStream_t st);
int launch_dispatch(const fcv2_fmt_t* fmt, const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E,
                    uint8_t* send, int32_t* expert_offsets, int32_t* row_src, void* ws, const Rec& rec, uint32_t row_bytes,
                    hipStream_t st);

// The checked dispatch call behind both C entry points (defined with the C ABI).
int dispatch_checked(const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E, const fcv2_fmt_t* fmt, void* send,
                     int32_t* expert_offsets, int32_t* row_src, void* ws, size_t ws_bytes, void* stream);

}  // namespace fcv2
