// fcv2_dispatch.hip -- fcv2_dispatch_quant: stable counting sort of the routed copies, then quantize-and-scatter (Sections 3.1, 4.4).
#include <atomic>

#include "fcv2_host.h"

namespace fcv2 {

// ---- dispatch: stable counting sort of the routed copies by expert, then quantize-and-scatter ------------------------
// Three launches, no order-dependent atomics, no waiting between blocks:
//   1. k_dispatch_count_rank   per chunk of 256 routed slots: the chunk's histogram over the experts, and for every slot
//                              its stable rank among the chunk's slots of the same expert (one byte);
//   2. k_dispatch_scan_chunks  per expert: exclusive prefix of the histograms over the chunks (in place) and the total;
//   3. the quantize-and-scatter kernel: every block scans the E totals itself (expert starts), forms the destination row
//      of each of its routed copies as start[e] + copies in earlier chunks + rank inside the chunk, and publishes
//      row_src (block 0 also expert_offsets) -- all of it while its tokens' loads are in flight.
// Ids outside [0, E) (including -1) are dropped slots.

// Exclusive prefix sum of one value per thread over a block of up to 8 waves; *total gets the block sum.
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t* lds8, int32_t* total) {
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = (blockDim.x + 63) >> 6;
    int32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t up = __shfl_up(inc, d);
        if ((int)lane >= d) inc += up;
    }
    if (lane == 63) lds8[wave] = inc;
    __syncthreads();
    int32_t before = 0, all = 0;
    for (uint32_t w = 0; w < n_waves; ++w) {
        const int32_t t = lds8[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    __syncthreads();
    return before + inc - v;
}

// Histogram of the chunk and stable in-chunk rank of every slot.  hist[chunk][e]; lrank[i] < 256.
// Every wave keeps, per expert, the 64-bit mask of its lanes that route to it (LDS integer OR: the result does not depend
// on the order of the lanes); a lane's rank inside the wave is the number of set bits below its own, the wave's count the
// number of set bits.  MASKS = false (more experts than the masks' LDS allows): the wave finds the lanes of each distinct
// expert with ballots instead, one round per distinct id.
template <bool MASKS>
__global__ __launch_bounds__(kChunk) void k_dispatch_count_rank(const int32_t* __restrict__ ids, uint32_t n_slots, uint32_t E,
                                                                int32_t* __restrict__ hist, uint8_t* __restrict__ lrank) {
    extern __shared__ uint32_t lds_cr[];  // MASKS: [kChunk/64][E][2] lane masks; else [kChunk/64][E] counts
    constexpr uint32_t kW = kChunk / 64;
    const uint32_t words = MASKS ? 2u : 1u;
    for (uint32_t t = threadIdx.x; t < kW * E * words; t += kChunk) lds_cr[t] = 0;
    __syncthreads();
    const uint32_t i = blockIdx.x * kChunk + threadIdx.x;
    const uint32_t wave = threadIdx.x / 64, lane = threadIdx.x & 63;
    int32_t e = -1;
    if (i < n_slots) {
        e = ids[i];
        if (e < 0 || (uint32_t)e >= E) e = -1;
    }
    uint32_t rank = 0;  // lanes below me in this wave with the same expert
    if (MASKS) {
        if (e >= 0) atomicOr(&lds_cr[(wave * E + (uint32_t)e) * 2 + (lane >> 5)], 1u << (lane & 31));
        __syncthreads();
        if (e >= 0) {
            uint32_t before = 0;
            for (uint32_t wv = 0; wv < wave; ++wv) before += __popc(lds_cr[(wv * E + e) * 2]) + __popc(lds_cr[(wv * E + e) * 2 + 1]);
            const uint32_t lo = lds_cr[(wave * E + e) * 2], hi = lds_cr[(wave * E + e) * 2 + 1];
            rank = lane < 32 ? __popc(lo & ((1u << lane) - 1u)) : __popc(lo) + __popc(hi & ((1u << (lane - 32)) - 1u));
            lrank[i] = (uint8_t)(before + rank);  // at most 255: a chunk has 256 slots
        }
        for (uint32_t t = threadIdx.x; t < E; t += kChunk) {
            int32_t c = 0;
#pragma unroll
            for (uint32_t wv = 0; wv < kW; ++wv) c += __popc(lds_cr[(wv * E + t) * 2]) + __popc(lds_cr[(wv * E + t) * 2 + 1]);
            hist[(uint64_t)blockIdx.x * E + t] = c;
        }
    } else {
        uint64_t todo = __ballot(e >= 0);
        while (todo) {  // one round per distinct expert id in the wave; every round clears at least one lane
            const int leader = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)todo) - 1);
            const int32_t el = __builtin_amdgcn_readlane(e, leader);  // a scalar read, not a trip through the LDS crossbar
            const uint64_t same = __ballot(e == el);
            if (e == el) {
                rank = __popcll(same & ((1ull << lane) - 1ull));
                if ((int)lane == leader) lds_cr[wave * E + el] = __popcll(same);
            }
            todo &= ~same;
        }
        __syncthreads();
        if (e >= 0) {
            uint32_t before = 0;
            for (uint32_t wv = 0; wv < wave; ++wv) before += lds_cr[wv * E + e];
            lrank[i] = (uint8_t)(before + rank);
        }
        for (uint32_t t = threadIdx.x; t < E; t += kChunk) {
            int32_t c = 0;
#pragma unroll
            for (uint32_t wv = 0; wv < kW; ++wv) c += (int32_t)lds_cr[wv * E + t];
            hist[(uint64_t)blockIdx.x * E + t] = c;
        }
    }
}

// One wave per expert: exclusive prefix over the chunks, in place; totals[e] = count of expert e.  A lane takes
// consecutive chunks; the scan across the lanes is a shuffle scan, so the kernel has no barrier.
__global__ __launch_bounds__(64) void k_dispatch_scan_chunks(int32_t* __restrict__ hist, uint32_t n_chunks, uint32_t E,
                                                             int32_t* __restrict__ totals) {
    const uint32_t e = blockIdx.x, lane = threadIdx.x;
    const uint32_t per = (n_chunks + 63) / 64;  // consecutive chunks per lane
    const uint32_t c0 = min(lane * per, n_chunks), c1 = min(c0 + per, n_chunks);
    int32_t s = 0;
    if (per <= 4) {  // up to 256 chunks (65,536 routed slots): four independent loads per lane
        int32_t v[4];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) v[k] = hist[(uint64_t)min(c0 + k, n_chunks - 1u) * E + e];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            if (c0 + k >= c1) v[k] = 0;
            s += v[k];
        }
        int32_t inc = s;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t up = __shfl_up(inc, d);
            if ((int)lane >= d) inc += up;
        }
        if (lane == 63) totals[e] = inc;
        int32_t run = inc - s;
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            if (c0 + k < c1) hist[(uint64_t)(c0 + k) * E + e] = run;
            run += v[k];
        }
    } else {
        for (uint32_t c = c0; c < c1; ++c) s += hist[(uint64_t)c * E + e];
        int32_t inc = s;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t up = __shfl_up(inc, d);
            if ((int)lane >= d) inc += up;
        }
        if (lane == 63) totals[e] = inc;
        int32_t run = inc - s;
        for (uint32_t c = c0; c < c1; ++c) {
            const int32_t v = hist[(uint64_t)c * E + e];
            hist[(uint64_t)c * E + e] = run;
            run += v;
        }
    }
}

// Expert starts (exclusive scan of the totals) into start[0..E), by the whole block, in two steps so that a caller can put
// other loads between them: the thread's share of the totals is read and summed first, the scan follows.  The second
// step returns the number of routed copies and ends with a barrier: start[] is complete for every thread.
struct StartsShare {
    uint32_t e0, e1;
    int32_t sum;
};
__device__ __forceinline__ StartsShare expert_starts_read(const int32_t* __restrict__ totals, uint32_t E) {
    const uint32_t per = (E + blockDim.x - 1) / blockDim.x;  // consecutive experts per thread
    StartsShare sh;
    sh.e0 = min(threadIdx.x * per, E);
    sh.e1 = min(sh.e0 + per, E);
    sh.sum = 0;
    for (uint32_t e = sh.e0; e < sh.e1; ++e) sh.sum += totals[e];
    return sh;
}
__device__ __forceinline__ int32_t expert_starts_scan(const StartsShare& sh, const int32_t* __restrict__ totals, int32_t* start, int32_t* lds8) {
    int32_t total;
    int32_t run = block_exclusive_scan(sh.sum, lds8, &total);
    for (uint32_t e = sh.e0; e < sh.e1; ++e) {
        start[e] = run;
        run += totals[e];
    }
    __syncthreads();
    return total;
}

// Destination row of routed slot i (or -1 for a dropped one) from the three planning results.
__device__ __forceinline__ int32_t dest_row_of(uint32_t i, const int32_t* __restrict__ ids, uint32_t E, const int32_t* __restrict__ hist,
                                               const uint8_t* __restrict__ lrank, const int32_t* start) {
    const int32_t e = ids[i];
    if (e < 0 || (uint32_t)e >= E) return -1;
    return start[e] + hist[(uint64_t)(i / kChunk) * E + e] + (int32_t)lrank[i];
}

// Only for row shapes the row-staged kernel cannot take: destination rows written out for the direct kernel.
__global__ __launch_bounds__(kChunk) void k_dispatch_dest(const int32_t* __restrict__ ids, uint32_t n_slots, uint32_t E,
                                                          const int32_t* __restrict__ hist, const int32_t* __restrict__ totals,
                                                          const uint8_t* __restrict__ lrank, int32_t* __restrict__ expert_offsets,
                                                          int32_t* __restrict__ dest, int32_t* __restrict__ row_src) {
    extern __shared__ int32_t start[];  // [E]
    __shared__ int32_t lds8[8];
    const int32_t total = expert_starts_scan(expert_starts_read(totals, E), totals, start, lds8);
    if (blockIdx.x == 0) {
        for (uint32_t e = threadIdx.x; e < E; e += kChunk) expert_offsets[e] = start[e];
        if (threadIdx.x == 0) expert_offsets[E] = total;
    }
    const uint32_t i = blockIdx.x * kChunk + threadIdx.x;
    if (i < n_slots) {
        const int32_t r = dest_row_of(i, ids, E, hist, lrank, start);
        dest[i] = r;
        if (r >= 0) row_src[r] = (int32_t)i;
    }
}

// ---- quantize-and-scatter -------------------------------------------------------------------------------------------
// Every token is quantized once and its packed row stored K times.  `rec` holds the row's section offsets (align 16).
// Rows are multiples of 32 elements, so a lane (32 consecutive elements) never straddles rows.
//
// What the copies cost is decided by how the stores meet the 128-byte lines of the send buffer: rows are 16-byte aligned
// only, so a store instruction that writes "this wave's piece of a plane" starts and ends inside lines, and metadata
// written by one lane in four touches a few bytes of each line.  The main kernel therefore assembles whole records in
// LDS and copies each to its K destinations as one contiguous run whose store instructions cover 8 whole lines each,
// with the non-temporal hint (measured on the MI355X, 65,536 copies, this kernel alone: 2-bit rows of 2,352 bytes
// 83 -> 58 us, 8-bit rows of 7,728 bytes 174 -> 119 us).  The direct kernel below it serves the shapes whose records do not fit.

// Lane's share of a record, written at `o` (the record's first byte, LDS or global) through `ST`.
template <int BITS, int LPG, bool SR, class ST>
__device__ __forceinline__ void put_lane(const ST& st, const Rec& rec, uint32_t r, uint32_t lig, uint32_t meta_mode, const uint32_t (&c)[8],
                                         const GroupMeta& m) {
    using P = Planes<BITS>;
    constexpr int U = 4;
    uint32_t q4[U], q2[U], q1 = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        q4[u] = P::w4 ? pack_plane4<P::sh4, BITS>(c[2 * u], c[2 * u + 1]) : 0u;
        q2[u] = P::w2 ? pack_plane2<P::sh2, BITS>(c[2 * u], c[2 * u + 1]) : 0u;
        if (P::w1) q1 |= pack_plane1<P::sh1, BITS>(c[2 * u], c[2 * u + 1]) << (8 * u);
    }
    if (P::w8) {
        st.halves(rec.plane8 + 32u * r, make_uint4(c[0], c[1], c[2], c[3]), make_uint4(c[4], c[5], c[6], c[7]));
    }
    if (P::w4) st.plane(rec.plane4 + 16u * r, make_uint4(q4[0], q4[1], q4[2], q4[3]));
    if (P::w2) st.plane(rec.plane2 + 8u * r, make_uint2(q2[0] | (q2[1] << 16), q2[2] | (q2[3] << 16)));
    if (P::w1) st.plane(rec.plane1 + 4u * r, q1);
    if (lig == 0) {
        const uint32_t g = r / LPG;
        if (meta_mode == kMetaInt) {
            st.meta(rec.scale + g, (uint8_t)m.raw_s);
            st.meta(rec.zero + g, (uint8_t)m.raw_z);
        } else if (meta_mode == kMetaFp32) {
            st.meta(rec.scale + 4u * g, m.s);
            st.meta(rec.zero + 4u * g, m.lo);
        } else {
            st.meta(rec.scale + 2u * g, (uint16_t)(f2u(m.s) >> 16));
            st.meta(rec.zero + 2u * g, (uint16_t)(f2u(m.lo) >> 16));
        }
        if (SR) {
            st.meta(rec.spike_val + 4u * g, m.sv);
            if (rec.idx_bf16)
                st.meta(rec.spike_idx + 4u * g, idx_pair_to_bf16(m.si));
            else
                st.meta(rec.spike_idx + 2u * g, (uint16_t)m.si);
        }
    }
}

struct PutLds {  // into a record staged in LDS
    uint8_t* o;
    template <class V> __device__ __forceinline__ void plane(uint32_t off, V v) const { *reinterpret_cast<V*>(o + off) = v; }
    template <class V> __device__ __forceinline__ void meta(uint32_t off, V v) const { *reinterpret_cast<V*>(o + off) = v; }
    __device__ __forceinline__ void halves(uint32_t off, uint4 a, uint4 b) const {
        plane(off, a);
        plane(off + 16u, b);
    }
};
template <bool NT_META> struct PutGlobal {  // straight into the send buffer
    uint8_t* o;
    template <class V> __device__ __forceinline__ void plane(uint32_t off, V v) const { store_stream(o + off, v); }
    template <class V> __device__ __forceinline__ void meta(uint32_t off, V v) const {
        if (NT_META) store_stream(o + off, v);
        else *reinterpret_cast<V*>(o + off) = v;
    }
    // a lane's 32 bytes of the 8-bit plane as two stores 32 bytes apart per lane: half lines, so no hint
    __device__ __forceinline__ void halves(uint32_t off, uint4 a, uint4 b) const {
        *reinterpret_cast<uint4*>(o + off) = a;
        *reinterpret_cast<uint4*>(o + off + 16u) = b;
    }
};

constexpr int kRowsBlockMax = 512;  // threads of the row-staged kernel (8 waves)

// Row-staged kernel.  A block owns `rows_per_block` consecutive tokens (blockDim = their lanes rounded up to whole waves,
// chosen on the host: the count up to 64 that leaves the fewest idle lanes; 1 and 2 rows measure the same at H = 7168).
// Dynamic LDS: per wave the transpose scratch | the records | the destination rows | the tables.
struct DispatchPlan {  // what the planning launches left in the workspace, and the two index outputs of the call
    const int32_t* ids;
    const int32_t* hist;
    const int32_t* totals;
    const uint8_t* lrank;
    int32_t* expert_offsets;
    int32_t* row_src;
    uint32_t E;
};

template <int BITS, int LPG, bool SR, bool INT_META>
__global__ __launch_bounds__(kRowsBlockMax) void k_dispatch_rows_t(const uint4* __restrict__ x, uint32_t T, uint32_t lanes_per_row,
                                                                  uint32_t K, DispatchPlan plan, uint8_t* __restrict__ send, Rec rec,
                                                                  uint32_t row_bytes, uint32_t meta_mode_arg, uint32_t rows_per_block) {
    // integer metadata is a compile-time variant, as in the quantize kernel: it would cost the float formats registers
    const uint32_t meta_mode = INT_META ? kMetaInt : (meta_mode_arg == kMetaFp32 ? kMetaFp32 : kMetaBf16);
    extern __shared__ uint4 smem[];
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint32_t n_waves = blockDim.x >> 6;
    uint4* scratch = smem + wave * (64 * kRowU4);
    uint4* recs = smem + n_waves * (64 * kRowU4);
    const uint32_t row_pieces = row_bytes >> 4;
    int32_t* drow = reinterpret_cast<int32_t*>(recs + rows_per_block * row_pieces);
    int32_t* start = drow + rows_per_block * K;
    float* tabs = reinterpret_cast<float*>(start + plan.E + 8);
    const uint32_t row0 = blockIdx.x * rows_per_block;
    const uint32_t rows_here = min(rows_per_block, T - row0);
    const uint32_t block_lanes = rows_here * lanes_per_row;
    // Planning, arranged so that nothing in it is waited for alone.  Loads return in the order they were issued: the
    // expert id of "my" routed slot and wave 0's share of the expert totals go out first, the tokens after them.  Wave 0
    // turns the totals into the expert starts (a scan inside one wave: no barrier of its own) while the tokens are on
    // their way; after the block's barrier the two gathers that complete a destination row are issued, and they arrive
    // while the tokens are being quantized.
    const uint32_t n_slots_here = rows_here * K;
    const uint32_t my_slot = row0 * K + threadIdx.x;
    // Both small reads are unconditional (clamped addresses, every wave) and looked at only after the tokens' loads are
    // out: a branch around a load, or a glance at its value, would make the wave wait for it right here.
    int32_t my_e = plan.ids[min(my_slot, T * K - 1u)];
    const uint32_t per = (plan.E + 63) / 64;  // consecutive experts per lane of wave 0
    const uint32_t e0 = min(lane * per, plan.E), e1 = min(e0 + per, plan.E);
    int32_t tot[4];  // up to 256 experts: the lane's totals, four independent loads
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) tot[k] = plan.totals[min(e0 + k, plan.E - 1u)];
    const bool has_tile = wave * 64 < block_lanes;  // whole waves past the block's last row only help with the copies
    TileIn in = {};
    if (has_tile) in = tile_load(x, (row0 * lanes_per_row + wave * 64) * 4, lane, (block_lanes - wave * 64) * 4);
    if (threadIdx.x >= n_slots_here) my_e = -1;
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k)
        if (per > 4 || e0 + k >= e1) tot[k] = 0;
    if (my_e < 0 || (uint32_t)my_e >= plan.E) my_e = -1;
    if (wave == 0) {
        int32_t my_sum = tot[0] + tot[1] + tot[2] + tot[3];
        if (per > 4)  // more than 256 experts: read in a loop (each read waited for; such routings are rare)
            for (uint32_t e = e0; e < e1; ++e) my_sum += plan.totals[e];
        int32_t inc = my_sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int32_t up = __shfl_up(inc, d);
            if ((int)lane >= d) inc += up;
        }
        int32_t run = inc - my_sum;
        if (per <= 4) {
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                if (e0 + k < e1) {
                    start[e0 + k] = run;
                    if (blockIdx.x == 0) plan.expert_offsets[e0 + k] = run;
                }
                run += tot[k];
            }
        } else {
            for (uint32_t e = e0; e < e1; ++e) {
                start[e] = run;
                if (blockIdx.x == 0) plan.expert_offsets[e] = run;
                run += plan.totals[e];
            }
        }
        if (blockIdx.x == 0 && lane == 63) plan.expert_offsets[plan.E] = inc;  // the last lane's inclusive sum: all routed copies
    }
    // the padding between a record's sections travels with the copies: it is written as zero
    for (uint32_t i = threadIdx.x; i < rows_here * row_pieces; i += blockDim.x) recs[i] = make_uint4(0, 0, 0, 0);
    if (INT_META) {
        for (uint32_t t = threadIdx.x; t < (uint32_t)kScaleTables; t += blockDim.x) tabs[t] = kScaleTablesInit.v[t];
    }
    __syncthreads();
    int32_t my_before = 0, my_rank = 0;
    if (my_e >= 0) {
        my_before = plan.hist[(uint64_t)(my_slot / kChunk) * plan.E + my_e];
        my_rank = (int32_t)plan.lrank[my_slot];
    }
    if (has_tile) {
        uint32_t w[16];
        tile_transpose(in, scratch, lane, w);
        const uint32_t l = wave * 64 + lane;
        uint32_t c[8];
        GroupMeta m;
        quantize_lane<BITS, kEplStream, LPG, SR>(w, lane & (LPG - 1), meta_mode, tabs, &scratch[lane * kRowU4], c, m);
        if (l < block_lanes) {
            const uint32_t rl = l / lanes_per_row;
            put_lane<BITS, LPG, SR>(PutLds{reinterpret_cast<uint8_t*>(recs + rl * row_pieces)}, rec, l - rl * lanes_per_row,
                                    lane & (LPG - 1), meta_mode, c, m);
        }
    }
    if (threadIdx.x < n_slots_here) {
        const int32_t r = my_e >= 0 ? start[my_e] + my_before + my_rank : -1;
        drow[threadIdx.x] = r;
        if (r >= 0) plan.row_src[r] = (int32_t)my_slot;
    }
    for (uint32_t i = threadIdx.x + blockDim.x; i < n_slots_here; i += blockDim.x) {  // more routed slots than threads: rare
        const uint32_t slot = row0 * K + i;
        const int32_t r = dest_row_of(slot, plan.ids, plan.E, plan.hist, plan.lrank, start);
        drow[i] = r;
        if (r >= 0) plan.row_src[r] = (int32_t)slot;
    }
    __syncthreads();
    // Copies.  One unit = 64 consecutive 16-byte pieces of one copy, cut so that a unit starts on a line of the send
    // buffer (the first unit of a copy starts up to 7 pieces before the record and masks them off).
    const uint32_t n_seg = (row_pieces + 7 + 63) >> 6;
    const uint32_t units = rows_here * K * n_seg;
    for (uint32_t u = wave; u < units; u += n_waves) {
        const uint32_t rk = u / n_seg, j = u - rk * n_seg;
        const int32_t d = drow[rk];
        if (d < 0) continue;
        const uint32_t ro = __umul24((uint32_t)d, row_bytes);  // 32-bit offsets: checked on the host
        const uint32_t a0 = (uint32_t)(reinterpret_cast<uintptr_t>(send) >> 4) + (ro >> 4);  // the copy's first piece, counted in pieces
        const uint32_t shift = a0 & 7u;
        const int32_t p = (int32_t)(j * 64 + lane) - (int32_t)shift;
        if (p >= 0 && (uint32_t)p < row_pieces) {
            const uint4 v = recs[(rk / K) * row_pieces + (uint32_t)p];
            uint8_t* at = send + (ro + 16u * (uint32_t)p);
            // The line a copy starts in and the line it ends in are shared with the neighbouring rows, which other blocks
            // write: those pieces go out as ordinary stores, so that the halves of such a line meet in the cache.
            const uint32_t line = (a0 + (uint32_t)p) >> 3, end = a0 + row_pieces;
            const bool shared = (shift != 0 && line == (a0 >> 3)) || ((end & 7u) != 0 && line == (end >> 3));
            if (shared) *reinterpret_cast<uint4*>(at) = v;
            else store_stream(at, v);
        }
    }
}

// Direct kernel: one wave tile = 2048 consecutive elements of x, every lane stores its share of the K copies itself.
template <int BITS, int LPG, bool SR, bool INT_META>
__global__ __launch_bounds__(kBlock) void k_dispatch_quant_t(const uint4* __restrict__ x, uint32_t n_lanes, uint32_t lanes_per_row,
                                                             uint32_t K, const int32_t* __restrict__ dest, uint8_t* __restrict__ send,
                                                             Rec rec, uint32_t row_bytes, uint32_t meta_mode_arg) {
    const uint32_t meta_mode = INT_META ? kMetaInt : (meta_mode_arg == kMetaFp32 ? kMetaFp32 : kMetaBf16);
    constexpr int EPL = kEplStream;
    __shared__ uint4 lds[kWaves][64 * kRowU4];
    __shared__ float tabs[kScaleTables];
    if (INT_META) fill_scale_tables(tabs);
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t lig = lane & (LPG - 1);
    const uint32_t tile = blockIdx.x * kWaves + wave;
    if (tile * 64 >= n_lanes) return;
    const TileIn cur = tile_load(x, (uint64_t)tile * 256, lane, n_lanes * 4 - tile * 256);
    uint32_t w[16];
    tile_transpose(cur, lds[wave], lane, w);
    const uint32_t L = tile * 64 + lane;
    if (L >= n_lanes) return;
    const uint32_t t = L / lanes_per_row;
    const uint32_t r = L - t * lanes_per_row;  // lane inside the row
    uint32_t c[EPL / 4];
    GroupMeta m;
    quantize_lane<BITS, EPL, LPG, SR>(w, lig, meta_mode, tabs, &lds[wave][lane * kRowU4], c, m);
    for (uint32_t k0 = 0; k0 < K; k0 += 8) {
        int32_t rows[8];  // all destinations first: the loads overlap instead of queueing one behind the other
#pragma unroll
        for (int i = 0; i < 8; ++i) rows[i] = (k0 + i < K) ? dest[t * K + k0 + i] : -1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (rows[i] < 0) continue;
            // the hint pays for metadata only where every lane stores (groups of 32)
            put_lane<BITS, LPG, SR>(PutGlobal<LPG == 1>{send + __umul24((uint32_t)rows[i], row_bytes)}, rec, r, lig, meta_mode, c, m);
        }
    }
}

static_assert(64 * kRowU4 * 16 == kWaveScratchBytes && kRowsBlockMax == kRowsPlanThreadsMax, "the launch plan and the kernel disagree");

template <int BITS, int G, bool SR> struct LaunchDispatch {
    static int run(const void* x, uint32_t T, uint32_t H, uint32_t K, const DispatchPlan& plan, int32_t* dest, uint8_t* send,
                   const Rec& rec, uint32_t row_bytes, uint32_t meta_mode, hipStream_t st) {
        constexpr int EPL = kEplStream, LPG = G / EPL;
        const uint32_t lpr = H / EPL, n_lanes = T * lpr;
        const bool im = meta_mode == kMetaInt;
        const RowsPlan rp = rows_plan(lpr, K, row_bytes, im, plan.E);
        if (rp.rows) {
            const dim3 grid((T + rp.rows - 1) / rp.rows), block(rp.threads);
            if (im)
                return launch(k_dispatch_rows_t<BITS, LPG, SR, true>, grid, block, rp.lds_bytes, st, (const uint4*)x, T, lpr, K, plan, send,
                              rec, row_bytes, meta_mode, rp.rows);
            return launch(k_dispatch_rows_t<BITS, LPG, SR, false>, grid, block, rp.lds_bytes, st, (const uint4*)x, T, lpr, K, plan, send, rec,
                          row_bytes, meta_mode, rp.rows);
        }
        // Row shapes the staged kernel cannot take: destination rows written out by one more small launch, then the direct kernel.
        const uint32_t n_slots = T * K;
        if (launch(k_dispatch_dest, dim3((n_slots + kChunk - 1) / kChunk), dim3(kChunk), plan.E * 4, st, plan.ids, n_slots, plan.E, plan.hist,
                   plan.totals, plan.lrank, plan.expert_offsets, dest, plan.row_src) != FCV2_OK)
            return FCV2_ERR_LAUNCH;
        const dim3 grid(grid_lanes(n_lanes)), block(kBlock);
        if (im)
            return launch(k_dispatch_quant_t<BITS, LPG, SR, true>, grid, block, 0, st, (const uint4*)x, n_lanes, lpr, K, (const int32_t*)dest,
                          send, rec, row_bytes, meta_mode);
        return launch(k_dispatch_quant_t<BITS, LPG, SR, false>, grid, block, 0, st, (const uint4*)x, n_lanes, lpr, K, (const int32_t*)dest, send,
                      rec, row_bytes, meta_mode);
    }
};

int launch_dispatch(const fcv2_fmt_t* fmt, const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E,
                    uint8_t* send, int32_t* expert_offsets, int32_t* row_src, void* ws, const Rec& rec, uint32_t row_bytes,
                    hipStream_t st) {
    const DispatchWs w = dispatch_ws(T, K, E);
    int32_t* hist = (int32_t*)((uint8_t*)ws + w.off_hist);
    int32_t* totals = (int32_t*)((uint8_t*)ws + w.off_totals);
    uint8_t* lrank = (uint8_t*)ws + w.off_lrank;
    int32_t* dest = (int32_t*)((uint8_t*)ws + w.off_dest);
    const size_t mask_bytes = (size_t)(kChunk / 64) * E * 8;  // lane masks per wave and expert: 8 KiB at 256 experts
    const int rc = mask_bytes <= 32 * 1024
                       ? launch(k_dispatch_count_rank<true>, dim3(w.n_chunks), dim3(kChunk), mask_bytes, st, ids, w.n_slots, E, hist, lrank)
                       : launch(k_dispatch_count_rank<false>, dim3(w.n_chunks), dim3(kChunk), mask_bytes / 2, st, ids, w.n_slots, E, hist, lrank);
    if (rc != FCV2_OK) return FCV2_ERR_LAUNCH;
    if (launch(k_dispatch_scan_chunks, dim3(E), dim3(64), 0, st, hist, w.n_chunks, E, totals) != FCV2_OK) return FCV2_ERR_LAUNCH;
    const DispatchPlan plan = {ids, hist, totals, lrank, expert_offsets, row_src, E};
    return by_format<LaunchDispatch>(fmt, x, T, H, K, plan, dest, send, rec, row_bytes, meta_mode_of(fmt), st);
}

}  // namespace fcv2

// ---- the dispatch call for callers that cannot allocate ------------------------------------------------------------
// The planning kernels' scratch (per-chunk histograms, expert totals, one destination row per slot) lives in a
// file-scope device array instead of a caller-supplied workspace.  Every GPU the library runs on holds its own copy of
// the array, at its own address, until the process ends.  In host code the array's name is only a stand-in for the
// device symbol: the address that kernels and copies need is asked of the runtime once per device
// (hipGetSymbolAddress, with that device current) and kept; host code below uses that pointer, never the name.
static __device__ __align__(256) uint8_t scratch[FCV2_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];  // zero-initialised; filled on the first call on each device

// Address of `scratch` on the current device, or nullptr (the runtime refused, or a device ordinal beyond kMaxDevices).
void* scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    // Two threads may both get here on a first call; both are told the same address, so the race is harmless.
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return nullptr;
    g_scratch_ptr[dev].store(q, std::memory_order_release);
    return q;
}
}  // namespace

extern "C" int fcv2_dispatch_quant_noalloc(const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E,
                                           const fcv2_fmt_t* fmt, void* send, int32_t* expert_offsets, int32_t* row_src, void* stream) {
    size_t need = 0;
    const int rc = fcv2_dispatch_workspace_bytes(T, K, E, &need);
    if (rc != FCV2_OK) return rc;
    if (need > (size_t)FCV2_STATIC_SCRATCH_BYTES) return FCV2_ERR_SCRATCH;  // the routing shape does not fit the static array
    void* ws = scratch_of_current_device();
    if (!ws) return FCV2_ERR_LAUNCH;
    // Nothing in the scratch has to start at zero: the counting kernel writes every histogram entry of every chunk, the
    // scan every total, the rank kernel every destination slot, before any of them is read.
    return fcv2::dispatch_checked(x, ids, T, H, K, E, fmt, send, expert_offsets, row_src, ws, FCV2_STATIC_SCRATCH_BYTES, stream);
}

