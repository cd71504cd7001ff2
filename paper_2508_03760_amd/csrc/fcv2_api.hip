// fcv2_api.hip -- the C ABI of libfcv2 (include/fcv2.h): argument checks and layout on the host, then the launch
// function of the call.  Also the plain copy kernel used as a bandwidth yardstick.
#include "fcv2_host.h"

namespace fcv2 {

// Plain streaming copy (16 bytes per lane), used to measure the practical HBM ceiling next to the codec kernels.
__global__ __launch_bounds__(kBlock) void k_stream_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, uint64_t n16) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n16) store_stream(&dst[i], src[i]);
}

static bool fmt_supported(const fcv2_fmt_t* f) {
    if (f->bits < 2 || f->bits > 8) return false;
    if (f->group != 32 && f->group != 64 && f->group != 128 && f->group != 256) return false;
    if ((f->flags & ~(FCV2_F_SPIKE | FCV2_F_META_FP32 | FCV2_F_META_INT | FCV2_F_IDX_BF16)) != 0) return false;
    if ((f->flags & FCV2_F_IDX_BF16) && !(f->flags & FCV2_F_SPIKE)) return false;  // index width means something only with spikes
    return (f->flags & (FCV2_F_META_FP32 | FCV2_F_META_INT)) != (FCV2_F_META_FP32 | FCV2_F_META_INT);  // one or the other
}


static Rec rec_of(const fcv2_layout_t& l, const fcv2_fmt_t* fmt) {
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
    r.idx_bf16 = (fmt->flags & FCV2_F_IDX_BF16) ? 1u : 0u;
    return r;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Largest tensor the kernels index with 32-bit offsets: 2^31 elements (a 4 GiB bf16 tensor).
static const uint64_t kMaxElems = 1ull << 31;

// Argument checks and launch of the dispatch call; serves both entry points (workspace from the caller, or the
// library's static scratch).
int dispatch_checked(const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E, const fcv2_fmt_t* fmt, void* send,
                     int32_t* expert_offsets, int32_t* row_src, void* ws, size_t ws_bytes, void* stream) {
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
    return launch_dispatch(fmt, x, ids, T, H, K, E, (uint8_t*)send, expert_offsets, row_src, ws, rec_of(l, fmt), (uint32_t)l.total_bytes,
                           (hipStream_t)stream);
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
        case FCV2_ERR_SCRATCH: return "routing shape exceeds the static scratch of the no-allocation entry point";
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
    out->off_spike_idx = take((fmt->flags & FCV2_F_SPIKE) != 0, ng * ((fmt->flags & FCV2_F_IDX_BF16) ? 4 : 2));
    out->total_bytes = round_up(off, align);  // the next record starts aligned too
    return FCV2_OK;
}

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
    return launch_quantize(fmt, x, n, packed, rec_of(l, fmt), n_slices, record_stride, (hipStream_t)stream);
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
    return launch_unpack(fmt, pp, n_slices, rec_of(l, fmt), n, out, (uint32_t)(out_dtype == FCV2_DT_FP32), (hipStream_t)stream);
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
    return launch_reduce(fmt_in, fmt_out, pp, n_peers, n, rec_of(lin, fmt_in), packed_out, rec_of(lout, fmt_out), sum_out, (hipStream_t)stream);
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
    return fcv2::dispatch_checked(x, ids, T, H, K, E, fmt, send, expert_offsets, row_src, ws, ws_bytes, stream);
}

int fcv2_stream_copy(const void* src, void* dst, uint64_t bytes, void* stream) {
    if (!src || !dst || bytes == 0 || bytes % 16 != 0) return FCV2_ERR_INVALID_ARG;
    if (!aligned16(src) || !aligned16(dst)) return FCV2_ERR_ALIGN;
    const uint64_t n16 = bytes / 16;
    return launch(k_stream_copy, dim3((unsigned)((n16 + kBlock - 1) / kBlock)), dim3(kBlock), 0, (hipStream_t)stream,
                  (const uint4*)src, (uint4*)dst, n16);
}

}  // extern "C"

