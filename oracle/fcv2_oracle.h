/*
 * fcv2_oracle.h -- C interface of the CPU oracle for the any-bit communication codec
 * (FlashCommunication V2, arxiv 2508.03760).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded reference written from the
 * paper's definitions.  It shares no code, header, table or helper with the HIP library: every
 * type and constant it needs is declared here again on purpose.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it; the product path never does.
 *
 * What each entry point follows:
 *   - asymmetric fine-grained round-to-nearest quantization per group      (Section 3.1)
 *   - bit splitting: a b-bit code stored as byte-aligned 4/2/1-bit planes   (Section 3.2, Fig. 3)
 *   - spike reserving: group min and max kept in float form with their
 *     in-group indices, the rest quantized over the shrunk range            (Section 3.3, Fig. 5)
 *   - metadata section sizes, spike indices as INT8 or as BF16 numbers      (Section 3.3, Table 4)
 *   - integer metadata: the scale as one byte, scale_int = round(log2(scale) * 10),
 *     and a one-byte zero                                                  (Section 3.3, Eq. 1, Table 4)
 *   - local dequantize-sum-requantize step of the two-step AllReduce        (Sections 3.1, 3.4)
 *   - dispatch-only quantization for MoE All2All                            (Section 3.1, 4.4)
 *
 * Pins (tests/test_oracle_*.py): Table 4 byte counts; sorted-order closed form and brute force for
 * the spike selection; exact spike restoration; |error| <= scale/2 bound; exhaustive plane
 * reassembly; reduction against float64 sums and special cases; a float64 textbook RTN quantizer
 * when spike reserving is off.  Parity unpinned by the paper (pinned only by this build's own
 * format statement and by round trips): which bits of a code go to which plane, the bit order
 * inside plane bytes, and the code value stored at spike positions.  The one-byte "zero" of Table 4's second row
 * is read as the textbook integer zero-point over a range widened to contain 0 (the table gives only its size):
 * the reading is unpinned by the paper, its arithmetic is pinned against the textbook affine quantizer.
 */
#ifndef FCV2_ORACLE_H
#define FCV2_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_OK = 0, ORC_ERR_ARG = -1 };
enum { ORC_F_SPIKE = 1u, ORC_F_META_FP32 = 2u, ORC_F_META_INT = 4u, ORC_F_IDX_BF16 = 8u };
enum { ORC_DT_BF16 = 0, ORC_DT_FP32 = 1 };

typedef struct {
    uint32_t bits;  /* 2..8 */
    uint32_t group; /* elements per quantization group, >= 3 (the library itself takes 32..256) */
    uint32_t flags; /* ORC_F_* */
} orc_fmt;

#define ORC_ABSENT UINT64_MAX

typedef struct {
    uint64_t n, n_groups, total_bytes;
    uint64_t off_plane8, off_plane4, off_plane2, off_plane1; /* ORC_ABSENT when the plane is not used */
    uint64_t off_scale, off_zero, off_spike_val, off_spike_idx;
} orc_layout;

/* Section offsets of one packed record of n elements; every section starts at a multiple of align and
 * total_bytes is rounded up to it. */
int orc_get_layout(uint64_t n, const orc_fmt* fmt, uint32_t align, orc_layout* out);

/* Order key of a bf16 bit pattern (total order, -0 < +0). */
uint32_t orc_key(uint16_t bf16_bits);

/* One group, no packing: writes codes[G], scale/zero as fp32 values actually stored, and (with
 * spike reserving) spike_val[2] raw bf16 bits and spike_idx[2].  Exposed so tests can pin the
 * quantizer separately from the wire format. */
int orc_quantize_group(const uint16_t* x, const orc_fmt* fmt, uint8_t* codes, float* scale, float* zero,
                       uint16_t* spike_val, uint8_t* spike_idx);

/* Integer metadata (ORC_F_META_INT).  Eq. 1 with theta = 10, clamped to a signed byte; its inverse
 * 2^(scale_int / 10) as an fp32 value; and both bytes of a group whose values to quantize span [lo, hi],
 * together with the scale s and the offset zf = -(zero_int * s) that a receiver reconstructs from them. */
int orc_scale_int(float scale);
float orc_scale_of_int(int scale_int);
int orc_meta_int(float lo, float hi, uint32_t bits, int8_t* scale_int, uint8_t* zero_int, float* s, float* zf);

/* Split n codes into the planes of `bits` and back (planes laid out with orc_get_layout(n, fmt, align)). */
int orc_split_pack(const uint8_t* codes, uint64_t n, const orc_fmt* fmt, uint32_t align, uint8_t* packed);
int orc_unpack_codes(const uint8_t* packed, uint64_t n, const orc_fmt* fmt, uint32_t align, uint8_t* codes);

int orc_quantize_pack(const uint16_t* x_bf16, uint64_t n, const orc_fmt* fmt, uint32_t align, uint8_t* packed);
int orc_unpack_dequant(const uint8_t* packed, uint64_t n, const orc_fmt* fmt, uint32_t align, void* out,
                       int out_dtype);
int orc_reduce_requant(const uint8_t* const* peers, int n_peers, uint64_t n, const orc_fmt* fmt_in,
                       const orc_fmt* fmt_out, uint32_t align, uint8_t* packed_out, float* sum_out_or_null);
/* Rows use align 16.  send_buf has R = number of ids != -1 rows of orc_get_layout(H, fmt, 16).total_bytes. */
int orc_dispatch_quant(const uint16_t* x_bf16, const int32_t* topk_ids, uint32_t T, uint32_t H, uint32_t K,
                       uint32_t E, const orc_fmt* fmt, uint8_t* send_buf, int32_t* expert_offsets,
                       int32_t* row_src);

/* fp32 -> bf16 round-to-nearest-even on bit patterns (NaN kept quiet). */
uint16_t orc_bf16_rne(float v);

#ifdef __cplusplus
}
#endif
#endif
