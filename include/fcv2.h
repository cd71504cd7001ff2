/*
 * fcv2.h -- C ABI of libfcv2: the any-bit quantize/pack codec of FlashCommunication V2
 * (arxiv 2508.03760) as hand-written HIP kernels for gfx950 (MI355X).
 *
 * The library squeezes collective payloads before transmission:
 *   - asymmetric fine-grained round-to-nearest quantization per group           (Section 3.1)
 *   - bit splitting: a b-bit code is stored as byte-aligned planes of 4, 2 and 1 bits
 *     (3 = 2+1, 5 = 4+1, 6 = 4+2, 7 = 4+2+1), each plane in a section of its own     (Section 3.2, Fig. 3)
 *   - spike reserving: the minimum and maximum of every group are kept as floats together with
 *     their in-group positions, and the rest is quantized over the shrunk range      (Section 3.3, Fig. 5)
 *
 * General rules for every call below
 *   - extern "C"; returns an FCV2_* status; never throws, never aborts, never synchronizes.
 *   - Pointers named *_dev are DEVICE pointers (HBM of the current HIP device); everything else is host memory.
 *   - The caller owns every buffer.  The library allocates no device memory and keeps no state between calls (no
 *     caches, no environment variables): a call depends on its arguments and on the current HIP device only.
 *   - FCV2_ERR_LAUNCH reports the status the runtime returned for this call's own launch; the runtime's "last error"
 *     slot is neither read nor cleared, so an error left there by other code of the process is not mistaken for ours.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the default stream); results are
 *     valid once the caller has synchronized that stream.
 *   - Device pointers must be 16-byte aligned (FCV2_ERR_ALIGN otherwise).
 *   - Inputs are finite bf16.  Non-finite values do not crash and give deterministic output.
 *   - A tensor call takes at most 2^31 elements (FCV2_ERR_UNSUPPORTED beyond), a dispatch call T*H <= 2^31.
 *
 * Packed record ("wire format") of n elements, as described by fcv2_get_layout():
 *     plane8 | plane4 | plane2 | plane1 | scale[ng] | zero[ng] | spike_val[2*ng] | spike_idx[2*ng]
 *   Quantized data first (regular part, then the extra-bit part), metadata after it (Fig. 3, Fig. 5c, Table 4).
 *   Every section starts at a multiple of `section_align` and total_bytes is rounded up to it, so records that
 *   follow each other stay aligned; absent sections have offset FCV2_ABSENT.
 *   The widest plane holds the most-significant bits of the code; inside a plane, elements are in natural
 *   order and the element with the lowest index occupies the least-significant bits of its byte.
 *   scale and zero are bf16 (fp32 with FCV2_F_META_FP32); zero is the float offset (the group's new minimum),
 *   spike_val[2g], spike_val[2g+1] are the raw bf16 bits of the group's min and max element, spike_idx the
 *   matching in-group positions as bytes.  The code stored at a spike position is 0.
 *   With FCV2_F_META_INT (Section 3.3, Eq. 1 and the second row of Table 4) scale and zero take one byte each:
 *   scale[g] is the signed byte scale_int = round(log2(scale) * 10), clamped to [-128, 127], and stands for the
 *   scale 2^(scale_int / 10) rounded to fp32; zero[g] is the unsigned zero-point round(-lo / scale) of the range
 *   widened to contain 0 and stands for the offset -(zero * scale); element = fma(code, scale, offset).
 *   Error bound with FCV2_F_META_INT: Eq. 1 rounds log2(scale) to the NEAREST tenth, so the decoded scale can be up to
 *   2^(1/20) (3.5 %) below the exact one; codes are clamped to [0, qmax], and a value at the top of the range is then off
 *   by up to (1/2 + 0.036 * qmax) steps instead of 1/2 (under 1 step up to 4 bits, about 9.7 steps at 8 bits); ranges
 *   wider than qmax * 2^12.7 or narrower than qmax * 2^-12.8 clip at the ends of the byte.  The mode is the paper's
 *   default for the low widths (Section 4.1: INT2 to INT4) and is accepted at every width for completeness.
 *   FCV2_F_META_FP32 and FCV2_F_META_INT exclude each other.
 *   With FCV2_F_IDX_BF16 (only together with FCV2_F_SPIKE) the spike positions are stored as BF16 numbers, two bytes each,
 *   instead of bytes: the first row of Table 4 (4096 INT2 values in groups of 32: 1024 + 512 + 512 + 512 = 2560 bytes;
 *   the default byte indices give 2304, byte indices with FCV2_F_META_INT the table's second row, 2048).
 */
#ifndef FCV2_H
#define FCV2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    FCV2_OK = 0,
    FCV2_ERR_INVALID_ARG = -1, /* null pointer, zero size, size not a multiple of the group, id out of range */
    FCV2_ERR_UNSUPPORTED = -2, /* bits outside 2..8, group not 32/64/128/256, unknown flag or flag pair, format pair not built */
    FCV2_ERR_ALIGN = -3,       /* a device pointer is not 16-byte aligned */
    FCV2_ERR_WORKSPACE = -4,   /* workspace smaller than fcv2_dispatch_workspace_bytes() */
    FCV2_ERR_LAUNCH = -5,      /* the HIP runtime refused the launch */
    FCV2_ERR_SCRATCH = -6      /* the shape needs more than the static scratch of the no-allocation entry point */
};

enum { FCV2_F_SPIKE = 1u, FCV2_F_META_FP32 = 2u, FCV2_F_META_INT = 4u, FCV2_F_IDX_BF16 = 8u };
enum { FCV2_DT_BF16 = 0, FCV2_DT_FP32 = 1 };

#define FCV2_ABSENT UINT64_MAX
#define FCV2_MAX_PEERS 16
#define FCV2_TENSOR_ALIGN 256u /* section alignment used by the tensor calls */
#define FCV2_ROW_ALIGN 16u     /* section alignment inside one dispatch row */

typedef struct {
    uint32_t bits;  /* 2..8 */
    uint32_t group; /* 32, 64, 128 or 256 elements per quantization group */
    uint32_t flags; /* FCV2_F_* */
} fcv2_fmt_t;

typedef struct {
    uint64_t n, n_groups, total_bytes;
    uint64_t off_plane8, off_plane4, off_plane2, off_plane1;
    uint64_t off_scale, off_zero, off_spike_val, off_spike_idx;
} fcv2_layout_t;

/* Section offsets and total size of one packed record (Table 4 gives the per-section byte counts: n*b/8 of
 * payload, one scale and one zero per group, one float value and one index per spike).  Host only, pure.
 * n > 0, n % group == 0, n % 8 == 0, section_align a power of two >= 1. */
int fcv2_get_layout(uint64_t n, const fcv2_fmt_t* fmt, uint32_t section_align, fcv2_layout_t* out);

/* Sender side (Sections 3.1-3.3): quantize n bf16 values group by group and write the packed record
 * (layout with FCV2_TENSOR_ALIGN) to packed_dev, which must hold total_bytes.  Padding between sections is
 * left untouched. */
int fcv2_quantize_pack(const void* x_bf16_dev, uint64_t n, const fcv2_fmt_t* fmt, void* packed_dev,
                       void* hip_stream);

/* Receiver side (Section 3.3): reassemble the codes, dequantize (code * scale + zero in one fused
 * multiply-add) and put the spikes back at their positions.  out_dev holds n values of out_dtype
 * (bf16: round-to-nearest-even; spike positions get the stored bits unchanged). */
int fcv2_unpack_dequant(const void* packed_dev, uint64_t n, const fcv2_fmt_t* fmt, void* out_dev, int out_dtype,
                        void* hip_stream);

/* The two exchanges of the two-step AllReduce (Sections 3.1, 3.4) move slices: rank r cuts its payload of n
 * elements into n_slices equal slices and sends slice j to rank j; after the local reduce every rank collects the
 * n_slices reduced slices.  These two calls are the sender and receiver sides with one launch each.
 *   fcv2_quantize_pack_slices: slice j of x becomes a packed record of n/n_slices elements at
 *     packed_dev + j * record_stride (record_stride >= that record's total_bytes, a multiple of 256).
 *   fcv2_unpack_dequant_slices: records_dev is a HOST array of n_slices DEVICE pointers, record j holds slice j
 *     of the output tensor of n elements.
 * 1 <= n_slices <= FCV2_MAX_PEERS; n % n_slices == 0; a slice is a whole number of groups and, for
 * n_slices > 1, a multiple of 2048 elements (FCV2_ERR_INVALID_ARG otherwise).  n_slices == 1 is the plain call. */
int fcv2_quantize_pack_slices(const void* x_bf16_dev, uint64_t n, uint32_t n_slices, const fcv2_fmt_t* fmt,
                              void* packed_dev, uint64_t record_stride, void* hip_stream);
int fcv2_unpack_dequant_slices(const void* const* records_dev, uint32_t n_slices, uint64_t n, const fcv2_fmt_t* fmt,
                               void* out_dev, int out_dtype, void* hip_stream);

/* Local step of the two-step quantized AllReduce (Sections 3.1, 3.4): dequantize the n_peers packed chunks
 * (all of format fmt_in, all resident in this GPU's memory), add them in fp32 in peer order 0..n_peers-1,
 * round the sum to bf16 and quantize it again with fmt_out into packed_out_dev.
 * peers_dev is a HOST array of n_peers DEVICE pointers (copied at call time), 1 <= n_peers <= FCV2_MAX_PEERS.
 * sum_out_dev, if not NULL, receives the n fp32 sums (before the bf16 rounding).
 * fmt_in and fmt_out must agree in group and FCV2_F_SPIKE (bits, the metadata flags and the index width may differ; equal
 * bits take a kernel specialised for the width, different bits one that switches on the input width at run time, a few
 * percent slower); other pairs give FCV2_ERR_UNSUPPORTED. */
int fcv2_reduce_requant(const void* const* peers_dev, int n_peers, uint64_t n, const fcv2_fmt_t* fmt_in,
                        const fcv2_fmt_t* fmt_out, void* packed_out_dev, float* sum_out_dev, void* hip_stream);

/* MoE dispatch (Section 3.1: only the dispatch volume is quantized; Section 4.4 measures it as an equal-split All2All;
 * grouping the routed copies per expert is what a real dispatch needs on top): quantize every token once
 * and write one packed row per routed copy into per-expert contiguous send buffers.
 *   x_bf16_dev    [T, H] bf16, H % group == 0
 *   topk_ids_dev  [T, K] int32, expert id in [0, E) or -1 for a dropped slot
 *   send_buf_dev  R rows of row_bytes = fcv2_get_layout(H, fmt, FCV2_ROW_ALIGN).total_bytes, R = number of
 *                 ids != -1 (the caller may size it for T*K rows); row_bytes is a multiple of 16; the padding
 *                 between a row's sections is written as zero or left untouched
 *   expert_offsets_dev [E+1] int32 out: expert e owns rows [expert_offsets[e], expert_offsets[e+1])
 *   row_src_dev   [T*K] int32 out: entry r < R is t*K+k of the copy stored in row r; inside an expert rows are
 *                 in ascending t*K+k (a stable counting sort)
 *   workspace_dev at least fcv2_dispatch_workspace_bytes(T, K, E) bytes of scratch, 16-byte aligned
 * Ids outside [-1, E) are treated as dropped: the call is asynchronous and cannot report what only the device sees
 * without a round trip to the host.  fcv2_dispatch_workspace_bytes gives the scratch size for a routing shape (counting
 * sort of T*K slots into E experts: per-chunk histograms, expert totals, one destination row per slot).  Limits (FCV2_ERR_UNSUPPORTED beyond): E <= 2048, T*K < 2^24,
 * T*K*row_bytes < 2^32 (a send buffer below 4 GiB). */
int fcv2_dispatch_workspace_bytes(uint32_t T, uint32_t K, uint32_t E, size_t* out);
int fcv2_dispatch_quant(const void* x_bf16_dev, const int32_t* topk_ids_dev, uint32_t T, uint32_t H, uint32_t K,
                        uint32_t E, const fcv2_fmt_t* fmt, void* send_buf_dev, int32_t* expert_offsets_dev,
                        int32_t* row_src_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* fcv2_dispatch_quant for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results, same kernels as
 * fcv2_dispatch_quant, but the planning scratch is a static device array inside the library (FCV2_STATIC_SCRATCH_BYTES
 * per GPU the library runs on, held until the process ends) instead of workspace_dev.  The call itself allocates
 * nothing and calls no allocating routine; the caller still passes the inputs and the three outputs.
 *   - A routing shape with fcv2_dispatch_workspace_bytes(T, K, E) > FCV2_STATIC_SCRATCH_BYTES gives FCV2_ERR_SCRATCH
 *     (2 MiB covers T*K = 131,072 routed slots over 256 experts, twice the DeepSeek-V3-shaped workload).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams,
 *     different threads) race on it and give wrong rows; calls on one stream, or ordered by events, are safe.  The
 *     array keeps the last call's contents; no call depends on them.
 *   - The first call on each device asks the runtime for the array's address (once per device; make that first call
 *     outside a graph capture). */
#define FCV2_STATIC_SCRATCH_BYTES (2u << 20)
int fcv2_dispatch_quant_noalloc(const void* x_bf16_dev, const int32_t* topk_ids_dev, uint32_t T, uint32_t H, uint32_t K,
                                uint32_t E, const fcv2_fmt_t* fmt, void* send_buf_dev, int32_t* expert_offsets_dev,
                                int32_t* row_src_dev, void* hip_stream);

/* Text for a status code (static storage, never NULL), and the version of this interface (major * 100 + minor).
 * House-keeping of the C ABI; they stand for nothing in the paper. */
const char* fcv2_status_string(int status);
int fcv2_version(void);

#ifdef __cplusplus
}
#endif
#endif
