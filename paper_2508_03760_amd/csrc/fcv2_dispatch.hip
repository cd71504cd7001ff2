// fcv2_dispatch.hip -- fcv2_dispatch_quant: stable counting sort of the routed copies, then quantize-and-scatter (Sections 3.1, 4.4).
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
        const int leader = __ffsll((unsigned long long)todo) - 1;
        const int32_t el = __shfl(e, leader);
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

// Quantize every token once, store the packed row K times.  `rec` holds the row's section offsets (align 16).
// One wave tile = 2048 consecutive elements of x (rows are multiples of 32 elements, so a lane never straddles rows).
template <int BITS, int LPG, bool SR>
__global__ __launch_bounds__(kBlock) void k_dispatch_quant_t(const uint4* __restrict__ x, uint32_t n_lanes, uint32_t lanes_per_row,
                                                             uint32_t K, const int32_t* __restrict__ dest, uint8_t* __restrict__ send,
                                                             Rec rec, uint32_t row_bytes, uint32_t meta_mode) {
    constexpr int EPL = kEplStream;
    __shared__ uint4 lds[kWaves][64 * kRowU4];
    __shared__ float tabs[kScaleTables];
    if (meta_mode == kMetaInt) fill_scale_tables(tabs);
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
    const uint32_t g = r / LPG;
    // The send buffer is addressed with 32-bit offsets (checked on the host): a row's offset is one 24-bit multiply,
    // every store one add on top of per-lane offsets computed once.
    using P = Planes<BITS>;
    constexpr int U = EPL / 8;
    uint32_t q4[U], q2[U], q1 = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        q4[u] = P::w4 ? pack_plane4<P::sh4, BITS>(c[2 * u], c[2 * u + 1]) : 0u;
        q2[u] = P::w2 ? (pack_plane2<P::sh2, BITS>(c[2 * u], c[2 * u + 1]) & 0xFFFFu) : 0u;
        if (P::w1) q1 |= (pack_plane1<P::sh1, BITS>(c[2 * u], c[2 * u + 1]) & 0xFFu) << (8 * u);
    }
    const uint32_t o8 = rec.plane8 + 32u * r, o4 = rec.plane4 + 16u * r, o2 = rec.plane2 + 8u * r, o1 = rec.plane1 + 4u * r;
    const uint32_t msz = (meta_mode == kMetaFp32) ? 4u : (meta_mode == kMetaInt) ? 1u : 2u;
    const uint32_t os = rec.scale + msz * g, oz = rec.zero + msz * g, ov = rec.spike_val + 4u * g, oi = rec.spike_idx + 2u * g;
    for (uint32_t k0 = 0; k0 < K; k0 += 8) {
        int32_t rows[8];  // all destinations first: the loads overlap instead of queueing one behind the other
#pragma unroll
        for (int i = 0; i < 8; ++i) rows[i] = (k0 + i < K) ? dest[t * K + k0 + i] : -1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (rows[i] < 0) continue;
            const uint32_t ro = __umul24((uint32_t)rows[i], row_bytes);
            if (P::w8) {
                *reinterpret_cast<uint4*>(send + (ro + o8)) = make_uint4(c[0], c[1], c[2], c[3]);
                *reinterpret_cast<uint4*>(send + (ro + o8 + 16u)) = make_uint4(c[4], c[5], c[6], c[7]);
            }
            if (P::w4) *reinterpret_cast<uint4*>(send + (ro + o4)) = make_uint4(q4[0], q4[1], q4[2], q4[3]);
            if (P::w2) *reinterpret_cast<uint2*>(send + (ro + o2)) = make_uint2(q2[0] | (q2[1] << 16), q2[2] | (q2[3] << 16));
            if (P::w1) *reinterpret_cast<uint32_t*>(send + (ro + o1)) = q1;
            if (lig == 0) {
                if (meta_mode == kMetaInt) {
                    send[ro + os] = (uint8_t)m.raw_s;
                    send[ro + oz] = (uint8_t)m.raw_z;
                } else if (meta_mode == kMetaFp32) {
                    *reinterpret_cast<float*>(send + (ro + os)) = m.s;
                    *reinterpret_cast<float*>(send + (ro + oz)) = m.lo;
                } else {
                    *reinterpret_cast<uint16_t*>(send + (ro + os)) = (uint16_t)(f2u(m.s) >> 16);
                    *reinterpret_cast<uint16_t*>(send + (ro + oz)) = (uint16_t)(f2u(m.lo) >> 16);
                }
                if (SR) {
                    *reinterpret_cast<uint32_t*>(send + (ro + ov)) = m.sv;
                    *reinterpret_cast<uint16_t*>(send + (ro + oi)) = (uint16_t)m.si;
                }
            }
        }
    }
}

template <int BITS, int G, bool SR> struct LaunchDispatch {
    static int run(const void* x, uint64_t n, uint32_t H, uint32_t K, const int32_t* dest, uint8_t* send, const Rec& rec,
                   uint32_t row_bytes, uint32_t meta_mode, hipStream_t st) {
        constexpr int EPL = kEplStream;
        const uint32_t n_lanes = (uint32_t)(n / EPL);
        hipLaunchKernelGGL((k_dispatch_quant_t<BITS, G / EPL, SR>), dim3(grid_lanes(n_lanes)), dim3(kBlock), 0, st,
                           (const uint4*)x, n_lanes, H / EPL, K, dest, send, rec, row_bytes, meta_mode);
        return launch_status();
    }
};

int launch_dispatch(const fcv2_fmt_t* fmt, const void* x, const int32_t* ids, uint32_t T, uint32_t H, uint32_t K, uint32_t E,
                    uint8_t* send, int32_t* expert_offsets, int32_t* row_src, void* ws, const Rec& rec, uint32_t row_bytes,
                    hipStream_t st) {
    const DispatchWs w = dispatch_ws(T, K, E);
    int32_t* hist = (int32_t*)((uint8_t*)ws + w.off_hist);
    int32_t* totals = (int32_t*)((uint8_t*)ws + w.off_totals);
    int32_t* dest = (int32_t*)((uint8_t*)ws + w.off_dest);
    hipLaunchKernelGGL(k_dispatch_count, dim3(w.n_chunks), dim3(kChunk), E * 4, st, ids, w.n_slots, E, hist);
    hipLaunchKernelGGL(k_dispatch_scan_chunks, dim3(E), dim3(256), 0, st, hist, w.n_chunks, E, totals);
    hipLaunchKernelGGL(k_dispatch_rank, dim3(w.n_chunks), dim3(kChunk), (kChunk / 64 + 1) * E * 4, st, ids, w.n_slots, E, hist,
                       (const int32_t*)totals, expert_offsets, dest, row_src);
    if (launch_status() != FCV2_OK) return FCV2_ERR_LAUNCH;
    return by_format<LaunchDispatch>(fmt, x, (uint64_t)T * H, H, K, (const int32_t*)dest, send, rec, row_bytes, meta_mode_of(fmt), st);
}

}  // namespace fcv2
