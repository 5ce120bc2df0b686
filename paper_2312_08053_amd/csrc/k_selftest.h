// Lane-exact checks of the wave primitives that are written with DPP operands (a wrong wait state or a
// folded operand shows as a wrong value in some lane, not as an error): one wave runs each of them on
// caller-given per-lane inputs and writes every lane's result out, for a test to compare with values
// computed on the host.
#pragma once
#include "common.h"
#include "k_alloc.h"
#include "k_alloc_band.h"

namespace kimad {

// out_u32: [0, 64) inclusive add-scan of in_u32 over the lanes;
//          [64 + (k4 * 4 + u) * 64 + lane] = in_u32[lane] + in_u32[64 + 16 * (lane / 16) + 4 * k4 + u]
//          (row_addr_sub4: the calling lane's base plus the second operand of lane K + u of its row of 16)
// out_f64: [(k4 * 4 + u) * 64 + lane] = in_f64[lane] + in_f64[64 + 16 * (lane / 16) + 4 * k4 + u]
//          (acc_rec_error4: the accumulator plus the error of lane K + u of the row)
//          [1024 + t * 64 + lane], t = 0, 1, 2: maximum of in_f64 over the lane's group of 2, 4, 8 lanes (group_max)
//          [1216 + t * 64 + lane], t = 0..3: the smallest in_f64 of the lane's group of 2, 4, 8, 16 lanes, and
// out_u32: [1088 + t * 64 + lane]: the smallest in_u32[64 + lane'] & 255 among the lanes of the group that hold it
//          (group_min_pair: the minimum of (value, record) pairs, the value first)
__global__ __launch_bounds__(64) void k_selftest_wave(const uint32_t* in_u32, const double* in_f64, uint32_t* out_u32,
                                                      double* out_f64) {
    const uint32_t lane = threadIdx.x;
    out_u32[lane] = wave_scan_add_u32(in_u32[lane]);
    const uint32_t base = in_u32[lane], second = in_u32[64 + lane];
    const double acc = in_f64[lane], err = in_f64[64 + lane];
    double one = 1.0;
    asm volatile("" : "+v"(one));
    uint32_t q[4];
    double t[4];
#define KIMAD_SELFTEST_K(K4)                                                                       \
    row_addr_sub4<4 * K4>(base, second, q);                                                        \
    t[0] = acc; t[1] = acc; t[2] = acc; t[3] = acc;                                                \
    acc_rec_error4<4 * K4>(t, err, one);                                                           \
    for (int u = 0; u < 4; ++u) {                                                                  \
        out_u32[64 + (K4 * 4 + u) * 64 + lane] = q[u];                                             \
        out_f64[(K4 * 4 + u) * 64 + lane] = t[u];                                                  \
    }
    KIMAD_SELFTEST_K(0)
    KIMAD_SELFTEST_K(1)
    KIMAD_SELFTEST_K(2)
    KIMAD_SELFTEST_K(3)
#undef KIMAD_SELFTEST_K
    out_f64[1024 + lane] = group_max<2>(acc);
    out_f64[1024 + 64 + lane] = group_max<4>(acc);
    out_f64[1024 + 128 + lane] = group_max<8>(acc);
    {
        double v;
        uint32_t k;
        v = acc; k = second & 255u; group_min_pair<2>(v, k); out_f64[1216 + lane] = v; out_u32[1088 + lane] = k;
        v = acc; k = second & 255u; group_min_pair<4>(v, k); out_f64[1216 + 64 + lane] = v; out_u32[1088 + 64 + lane] = k;
        v = acc; k = second & 255u; group_min_pair<8>(v, k); out_f64[1216 + 128 + lane] = v; out_u32[1088 + 128 + lane] = k;
        v = acc; k = second & 255u; group_min_pair<16>(v, k); out_f64[1216 + 192 + lane] = v; out_u32[1088 + 192 + lane] = k;
    }
}

}  // namespace kimad
