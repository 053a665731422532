// Dequantizer in the rotated domain (section 2.1: X^ = round(X / Delta) * Delta): packed b-bit codes
// and their scales back to floating-point values, without a rotation.  y^_j = code_j * Delta for the
// signed per-token codes, code_j * Delta_g + lo_g for the unsigned group-128 codes (section 5.1).
// One thread takes 8 codes (b bytes of the row's bit stream) and writes 8 floats.
#include "rotq_internal.h"

namespace rq {
namespace {

constexpr int kThreads = 256;

template <int BITS, bool ASYM>
__global__ __launch_bounds__(kThreads) void k_dequantize(const uint8_t* codes, const float* scales,
                                                         const float* mins, int64_t rows, int n, float* Y,
                                                         bool y16) {
    const int gpr = n >> 3;                                  // groups of 8 codes per row
    const int64_t total = rows * gpr;
    for (int64_t it = (int64_t)blockIdx.x * kThreads + threadIdx.x; it < total; it += (int64_t)gridDim.x * kThreads) {
        const int64_t row = it / gpr;
        const int grp = (int)(it - row * gpr);
        const uint8_t* p = codes + row * ((int64_t)n * BITS / 8) + grp * BITS;
        uint32_t w = 0;
#pragma unroll
        for (int k = 0; k < BITS; ++k) w |= (uint32_t)p[k] << (8 * k);
        float delta, lo = 0.0f;
        if constexpr (ASYM) {
            const int64_t gi = row * (n / RQ_GROUP) + (grp * 8) / RQ_GROUP;
            delta = scales[gi];
            lo = mins[gi];
        } else {
            delta = scales[row];
        }
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t f = (w >> (BITS * k)) & ((1u << BITS) - 1u);
            if constexpr (ASYM) {
                v[k] = fmaf((float)f, delta, lo);
            } else {
                const int q = (int)(f ^ (1u << (BITS - 1))) - (1 << (BITS - 1));   // two's complement field
                v[k] = (float)q * delta;
            }
        }
        float* out = Y + row * (int64_t)n + grp * 8;
        if (y16) {
            reinterpret_cast<float4*>(out)[0] = make_float4(v[0], v[1], v[2], v[3]);
            reinterpret_cast<float4*>(out)[1] = make_float4(v[4], v[5], v[6], v[7]);
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) out[k] = v[k];
        }
    }
}

}  // namespace

int dequantize_rows(const uint32_t* codes, const float* scales, const float* mins, int64_t rows, int n, int bits,
                    float* Y, hipStream_t s) {
    const int64_t total = rows * (n >> 3);
    const int64_t want = (total + kThreads - 1) / kThreads;
    const unsigned grid = (unsigned)(want < (1 << 20) ? want : (1 << 20));
    const bool y16 = (reinterpret_cast<uintptr_t>(Y) & 15) == 0;     // rows are n * 4 bytes, n a multiple of 8
    const uint8_t* c = reinterpret_cast<const uint8_t*>(codes);
    if (mins) {
        if (bits == 4) hipLaunchKernelGGL((k_dequantize<4, true>), dim3(grid), dim3(kThreads), 0, s, c, scales, mins, rows, n, Y, y16);
        else hipLaunchKernelGGL((k_dequantize<3, true>), dim3(grid), dim3(kThreads), 0, s, c, scales, mins, rows, n, Y, y16);
    } else {
        if (bits == 4) hipLaunchKernelGGL((k_dequantize<4, false>), dim3(grid), dim3(kThreads), 0, s, c, scales, mins, rows, n, Y, y16);
        else hipLaunchKernelGGL((k_dequantize<3, false>), dim3(grid), dim3(kThreads), 0, s, c, scales, mins, rows, n, Y, y16);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace rq
