// fcv2_dispatch.hip -- fcv2_dispatch_quant: stable counting sort of the routed copies, then quantize-and-scatter (Sections 3.1, 4.4).
#include <atomic>

#include "fcv2_host.h"

namespace fcv2 {

// ---- dispatch: stable counting sort of the routed copies by expert, then quantize-and-scatter ------------------------

// Per-chunk histogram of expert ids.  hist[chunk][e].
__global__ __launch_bounds__(kChunk) void k_dispatch_count(const int32_t* __restrict__ ids, uint32_t n_slots, uint32_t E,
                                                           int32_t* __restrict__ hist) {
    extern __shared__ int32_t lds[];
    for (uint32_t e = threadIdx.x; e < E; e += kChunk) lds[e] = 0;
    __syncthreads();
    const uint32_t i = blockIdx.x * kChunk + threadIdx.x;
    if (i < n_slots) {
        const int32_t e = ids[i];
        if (e >= 0 && (uint32_t)e < E) atomicAdd(&lds[e], 1);  // integer counts: order does not matter
    }
    __syncthreads();
    for (uint32_t e = threadIdx.x; e < E; e += kChunk) hist[(uint64_t)blockIdx.x * E + e] = lds[e];
}

// Exclusive prefix sum of one value per thread over a block of 256 threads; *total gets the block sum.
__device__ __forceinline__ int32_t block_exclusive_scan_256(int32_t v, int32_t* lds4, int32_t* total) {
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int32_t up = __shfl_up(inc, d);
        if ((int)lane >= d) inc += up;
    }
    if (lane == 63) lds4[wave] = inc;
    __syncthreads();
    int32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int32_t t = lds4[w];
        if ((uint32_t)w < wave) before += t;
        all += t;
    }
    *total = all;
    __syncthreads();
    return before + inc - v;
}

// One block per expert: exclusive prefix over the chunks, in place; totals[e] = count of expert e.
__global__ __launch_bounds__(256) void k_dispatch_scan_chunks(int32_t* __restrict__ hist, uint32_t n_chunks, uint32_t E,
                                                              int32_t* __restrict__ totals) {
    __shared__ int32_t lds4[4];
    const uint32_t e = blockIdx.x;
    const uint32_t per = (n_chunks + 255) / 256;  // consecutive chunks per thread
    const uint32_t c0 = threadIdx.x * per, c1 = min(c0 + per, n_chunks);
    int32_t s = 0;
    for (uint32_t c = c0; c < c1; ++c) s += hist[(uint64_t)c * E + e];
    int32_t total;
    int32_t run = block_exclusive_scan_256(s, lds4, &total);
    if (threadIdx.x == 0) totals[e] = total;
    for (uint32_t c = c0; c < c1; ++c) {
        const int32_t v = hist[(uint64_t)c * E + e];
        hist[(uint64_t)c * E + e] = run;
        run += v;
    }
}

// Destination row of every routed slot: expert start + copies in earlier chunks + copies earlier in this chunk.
// Every block derives the expert starts (exclusive scan of the totals) itself; block 0 also publishes them.
__global__ __launch_bounds__(kChunk) void k_dispatch_rank(const int32_t* __restrict__ ids, uint32_t n_slots, uint32_t E,
                                                          const int32_t* __restrict__ hist, const int32_t* __restrict__ totals,
                                                          int32_t* __restrict__ expert_offsets, int32_t* __restrict__ dest,
                                                          int32_t* __restrict__ row_src) {
    extern __shared__ int32_t lds[];  // [kChunk/64][E] copies of expert e in each wave of this chunk, then [E] expert starts
    __shared__ int32_t lds4[4];
    constexpr int kW = kChunk / 64;
    int32_t* start = lds + kW * E;
    for (uint32_t t = threadIdx.x; t < kW * E; t += kChunk) lds[t] = 0;
    {   // expert starts: consecutive experts per thread, block scan of the per-thread sums
        const uint32_t per = (E + kChunk - 1) / kChunk;
        const uint32_t e0 = threadIdx.x * per, e1 = min(e0 + per, E);
        int32_t s = 0;
        for (uint32_t e = e0; e < e1; ++e) s += totals[e];
        int32_t total;
        int32_t run = block_exclusive_scan_256(s, lds4, &total);
        for (uint32_t e = e0; e < e1; ++e) {
            start[e] = run;
            if (blockIdx.x == 0) expert_offsets[e] = run;
            run += totals[e];
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) expert_offsets[E] = total;
    }
    __syncthreads();
    const uint32_t i = blockIdx.x * kChunk + threadIdx.x;
    const uint32_t wave = threadIdx.x / 64, lane = threadIdx.x & 63;
    int32_t e = -1;
    if (i < n_slots) {
        e = ids[i];
        if (e < 0 || (uint32_t)e >= E) e = -1;
    }
    // stable rank inside the wave: lanes below me with the same expert
    uint32_t rank = 0;
    uint64_t todo = __ballot(e >= 0);
    while (todo) {  // one round per distinct expert id in the wave; every round clears at least one lane
        const int leader = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)todo) - 1);
        const int32_t el = __builtin_amdgcn_readlane(e, leader);  // a scalar read, not a trip through the LDS crossbar
        const uint64_t same = __ballot(e == el);
        if (e == el) {
            rank = __popcll(same & ((1ull << lane) - 1ull));
            if ((int)lane == leader) lds[wave * E + el] = __popcll(same);
        }
        todo &= ~same;
    }
    __syncthreads();
    if (e >= 0) {
        uint32_t before = 0;
        for (uint32_t wv = 0; wv < wave; ++wv) before += lds[wv * E + e];
        const int32_t r = start[e] + hist[(uint64_t)blockIdx.x * E + e] + (int32_t)(before + rank);
        dest[i] = r;
        row_src[r] = (int32_t)i;
    } else if (i < n_slots) {
        dest[i] = -1;
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
// with the non-temporal hint (measured on the MI355X, 65,536 copies: 2-bit rows of 2,352 bytes 83 -> 58 us for the whole
// call, 8-bit rows of 7,728 bytes 174 -> 119 us).  The direct kernel below it serves the shapes whose records do not fit.

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
template <int BITS, int LPG, bool SR, bool INT_META>
__global__ __launch_bounds__(kRowsBlockMax) void k_dispatch_rows_t(const uint4* __restrict__ x, uint32_t T, uint32_t lanes_per_row,
                                                                  uint32_t K, const int32_t* __restrict__ dest,
                                                                  uint8_t* __restrict__ send, Rec rec, uint32_t row_bytes,
                                                                  uint32_t meta_mode_arg, uint32_t rows_per_block) {
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
    float* tabs = reinterpret_cast<float*>(drow + rows_per_block * K);
    const uint32_t row0 = blockIdx.x * rows_per_block;
    const uint32_t rows_here = min(rows_per_block, T - row0);
    const uint32_t block_lanes = rows_here * lanes_per_row;
    for (uint32_t i = threadIdx.x; i < rows_here * K; i += blockDim.x) drow[i] = dest[row0 * K + i];
    // the padding between a record's sections travels with the copies: it is written as zero
    for (uint32_t i = threadIdx.x; i < rows_here * row_pieces; i += blockDim.x) recs[i] = make_uint4(0, 0, 0, 0);
    if (INT_META) {
        for (uint32_t t = threadIdx.x; t < (uint32_t)kScaleTablePow; t += blockDim.x) tabs[t] = scale_table_pow((int)t);
        for (uint32_t t = threadIdx.x; t < (uint32_t)kScaleTableThr; t += blockDim.x) tabs[kScaleTablePow + t] = scale_table_thr((int)t);
    }
    __syncthreads();
    if (wave * 64 < block_lanes) {  // whole waves past the block's last row only help with the copies
        const uint32_t piece0 = (row0 * lanes_per_row + wave * 64) * 4;
        const TileIn in = tile_load(x, piece0, lane, (block_lanes - wave * 64) * 4);
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
    static int run(const void* x, uint32_t T, uint32_t H, uint32_t K, const int32_t* dest, uint8_t* send, const Rec& rec,
                   uint32_t row_bytes, uint32_t meta_mode, hipStream_t st) {
        constexpr int EPL = kEplStream, LPG = G / EPL;
        const uint32_t lpr = H / EPL, n_lanes = T * lpr;
        const bool im = meta_mode == kMetaInt;
        const RowsPlan plan = rows_plan(lpr, K, row_bytes, im);
        if (plan.rows) {
            const dim3 grid((T + plan.rows - 1) / plan.rows), block(plan.threads);
            if (im)
                return launch(k_dispatch_rows_t<BITS, LPG, SR, true>, grid, block, plan.lds_bytes, st, (const uint4*)x, T, lpr, K, dest,
                              send, rec, row_bytes, meta_mode, plan.rows);
            return launch(k_dispatch_rows_t<BITS, LPG, SR, false>, grid, block, plan.lds_bytes, st, (const uint4*)x, T, lpr, K, dest, send,
                          rec, row_bytes, meta_mode, plan.rows);
        }
        const dim3 grid(grid_lanes(n_lanes)), block(kBlock);
        if (im)
            return launch(k_dispatch_quant_t<BITS, LPG, SR, true>, grid, block, 0, st, (const uint4*)x, n_lanes, lpr, K, dest, send, rec,
                          row_bytes, meta_mode);
        return launch(k_dispatch_quant_t<BITS, LPG, SR, false>, grid, block, 0, st, (const uint4*)x, n_lanes, lpr, K, dest, send, rec,
                      row_bytes, meta_mode);
    }
};


int launch_dispatch(const fcv2_fmt_t* fmt, const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E,
                    uint8_t* send, int32_t* expert_offsets, int32_t* row_src, void* ws, const Rec& rec, uint32_t row_bytes,
                    hipStream_t st) {
    const DispatchWs w = dispatch_ws(T, K, E);
    int32_t* hist = (int32_t*)((uint8_t*)ws + w.off_hist);
    int32_t* totals = (int32_t*)((uint8_t*)ws + w.off_totals);
    int32_t* dest = (int32_t*)((uint8_t*)ws + w.off_dest);
    if (launch(k_dispatch_count, dim3(w.n_chunks), dim3(kChunk), E * 4, st, ids, w.n_slots, E, hist) != FCV2_OK) return FCV2_ERR_LAUNCH;
    if (launch(k_dispatch_scan_chunks, dim3(E), dim3(256), 0, st, hist, w.n_chunks, E, totals) != FCV2_OK) return FCV2_ERR_LAUNCH;
    if (launch(k_dispatch_rank, dim3(w.n_chunks), dim3(kChunk), (kChunk / 64 + 1) * E * 4, st, ids, w.n_slots, E, (const int32_t*)hist,
               (const int32_t*)totals, expert_offsets, dest, row_src) != FCV2_OK)
        return FCV2_ERR_LAUNCH;
    return by_format<LaunchDispatch>(fmt, x, T, H, K, (const int32_t*)dest, send, rec, row_bytes, meta_mode_of(fmt), st);
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

