// fcv2_hostcheck.cpp -- host build of the kernels' integer/float building blocks (fcv2_bits.h) behind a C
// interface, so that the CPU test suite can exercise exactly the sequences the kernels run.
// Build: g++ -std=c++17 -O2 -ffp-contract=off -fPIC -shared.
#include <cstring>

#include "../../paper_2508_03760_amd/csrc/fcv2_bits.h"

using namespace fcv2;

template <int BITS> static void planes_of_codes(const uint8_t* codes, uint32_t* p8lo, uint32_t* p8hi, uint32_t* p4, uint32_t* p2,
                                                uint32_t* p1) {
    uint32_t c0, c1;
    std::memcpy(&c0, codes, 4);
    std::memcpy(&c1, codes + 4, 4);
    using P = Planes<BITS>;
    *p8lo = c0;
    *p8hi = c1;
    *p4 = P::w4 ? pack_plane4<P::sh4, BITS>(c0, c1) : 0;
    *p2 = P::w2 ? pack_plane2<P::sh2, BITS>(c0, c1) : 0;  // must come back with nothing above bit 15
    *p1 = P::w1 ? pack_plane1<P::sh1, BITS>(c0, c1) : 0;    // nothing above bit 7
}

template <int BITS> static void codes_of_planes(uint32_t p4, uint32_t p2, uint32_t p1, uint8_t* codes) {
    uint32_t ev, od;
    codes_even_odd<BITS>(p4, p2, p1, ev, od);
    for (int i = 0; i < 4; ++i) {
        codes[2 * i] = (uint8_t)(ev >> (8 * i));
        codes[2 * i + 1] = (uint8_t)(od >> (8 * i));
    }
}

template <int BITS> static void pairs_of_planes(uint32_t p8lo, uint32_t p8hi, uint32_t p4, uint32_t p2, uint32_t p1, uint8_t* codes) {
    uint32_t Q[4];
    codes_pairs<BITS>(p8lo, p8hi, p4, p2, p1, Q);
    for (int k = 0; k < 4; ++k) {
        codes[k] = (uint8_t)(Q[k] & 0xFFFFu);
        codes[k + 4] = (uint8_t)(Q[k] >> 16);
        if ((Q[k] & 0xFF00FF00u) != 0) codes[k] = 0xEE;  // must be zero-extended
    }
}

// 16 codes from the masked-in-place pair registers: every half must be code << pos with nothing else set.
template <int BITS> static int pairs16_of_planes(uint32_t p4a, uint32_t p4b, uint32_t p2, uint32_t p1, uint8_t* codes) {
    uint32_t Q[8];
    codes_pairs16<BITS>(p4a, p4b, p2, p1, Q);
    using M = PairMap<BITS>;
    for (int e = 0; e < 16; ++e) codes[e] = 0xEE;
    for (int k = 0; k < 8; ++k) {
        const uint32_t l = Q[k] & 0xFFFFu, h = Q[k] >> 16;
        const uint32_t field = ((1u << BITS) - 1u) << M::pos(k);
        if ((l & ~field) || (h & ~field) || M::pos(k) + BITS > 10) return -2;
        codes[M::lo(k)] = (uint8_t)(l >> M::pos(k));
        codes[M::hi(k)] = (uint8_t)(h >> M::pos(k));
    }
    return 0;
}

template <int QMAX> static uint64_t div_mismatches(uint32_t first_bits, uint32_t count) {
    uint64_t bad = 0;
    for (uint32_t i = 0; i < count; ++i) {
        uint32_t u = first_bits + i;
        float d;
        std::memcpy(&d, &u, 4);
        float a = div_by_qmax<QMAX>(d), b = d / (float)QMAX;
        if (std::memcmp(&a, &b, 4) != 0 && !(a != a && b != b)) ++bad;
    }
    return bad;
}

extern "C" {

int hc_planes_of_codes(int bits, const uint8_t* codes, uint32_t* out5) {
    switch (bits) {
#define C(B) case B: planes_of_codes<B>(codes, out5, out5 + 1, out5 + 2, out5 + 3, out5 + 4); return 0;
        C(2) C(3) C(4) C(5) C(6) C(7) C(8)
#undef C
    }
    return -1;
}

int hc_codes_of_planes(int bits, uint32_t p4, uint32_t p2, uint32_t p1, uint8_t* codes) {
    switch (bits) {
#define C(B) case B: codes_of_planes<B>(p4, p2, p1, codes); return 0;
        C(2) C(3) C(4) C(5) C(6) C(7)
#undef C
    }
    return -1;
}

int hc_pairs_of_planes(int bits, uint32_t p8lo, uint32_t p8hi, uint32_t p4, uint32_t p2, uint32_t p1, uint8_t* codes) {
    switch (bits) {
#define C(B) case B: pairs_of_planes<B>(p8lo, p8hi, p4, p2, p1, codes); return 0;
        C(2) C(3) C(4) C(5) C(6) C(7) C(8)
#undef C
    }
    return -1;
}

int hc_pairs16_of_planes(int bits, uint32_t p4a, uint32_t p4b, uint32_t p2, uint32_t p1, uint8_t* codes) {
    switch (bits) {
        case 2: return pairs16_of_planes<2>(p4a, p4b, p2, p1, codes);
        case 3: return pairs16_of_planes<3>(p4a, p4b, p2, p1, codes);
        case 4: return pairs16_of_planes<4>(p4a, p4b, p2, p1, codes);
    }
    return -1;
}

// Number of fp32 bit patterns in [first_bits, first_bits + count) where the short division differs from d / qmax.
uint64_t hc_div_mismatches(int qmax, uint32_t first_bits, uint32_t count) {
    switch (qmax) {
#define C(Q) case Q: return div_mismatches<Q>(first_bits, count);
        C(3) C(7) C(15) C(31) C(63) C(127) C(255)
#undef C
    }
    return ~0ull;
}

// Integer scale (Eq. 1) of `count` fp32 bit patterns starting at first_bits: k[i] and the bits of 2^(k/10).
void hc_scale_int_of(uint32_t first_bits, uint32_t count, int8_t* k, uint32_t* s_bits) {
    for (uint32_t i = 0; i < count; ++i) {
        const uint32_t b = first_bits + i;
        float f;
        memcpy(&f, &b, 4);
        const ScaleInt r = scale_int_of(f);
        k[i] = (int8_t)r.k;
        memcpy(&s_bits[i], &r.s, 4);
    }
}
// Entries of the compile-time tables that differ (as bit patterns) from what the table functions compute.
int hc_scale_tables_mismatches() {
    int bad = 0;
    for (int t = 0; t < kScaleTablePow + kScaleTableThr; ++t) {
        const float want = t < kScaleTablePow ? scale_table_pow(t) : scale_table_thr(t - kScaleTablePow);
        bad += memcmp(&want, &kScaleTablesInit.v[t], 4) != 0;
    }
    return bad;
}
// The same through the per-code tables.
void hc_scale_int_from_tables(uint32_t first_bits, uint32_t count, int8_t* k, uint32_t* s_bits) {
    const float* pow_tab = kScaleTablesInit.v;  // the compile-time tables, as the kernels copy them into LDS
    const float* thr_tab = kScaleTablesInit.v + kScaleTablePow;
    for (uint32_t i = 0; i < count; ++i) {
        const uint32_t b = first_bits + i;
        float f;
        memcpy(&f, &b, 4);
        const ScaleInt r = scale_int_from_tables(f, pow_tab, thr_tab);
        k[i] = (int8_t)r.k;
        memcpy(&s_bits[i], &r.s, 4);
    }
}
int hc_scale_int_estimate(float s) { return scale_int_estimate(s); }
float hc_scale_of_int(int k) { return scale_of_int(k); }

// Launch plan of the row-staged dispatch kernel: out3 = {rows per block, threads, LDS bytes}.
void hc_rows_plan(uint32_t lpr, uint32_t K, uint32_t row_bytes, int int_meta, uint32_t E, uint64_t* out3) {
    const RowsPlan p = rows_plan(lpr, K, row_bytes, int_meta != 0, E);
    out3[0] = p.rows;
    out3[1] = p.threads;
    out3[2] = p.lds_bytes;
}

uint32_t hc_key_of_bf16(uint32_t u) { return key_of_bf16(u); }
uint32_t hc_bf16_of_key(uint32_t k) { return bf16_of_key(k); }
uint32_t hc_bf16_rne_bits(uint32_t u) { return bf16_rne_bits(u); }
uint32_t hc_bf16_round_up_bits(uint32_t u) { return bf16_round_up_bits(u); }
}
