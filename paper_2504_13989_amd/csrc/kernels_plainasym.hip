// Rotation-free asymmetric quantizer in groups of 128 values (section 5.1, the KV-cache setting, for
// a tensor whose rotation is fused into the producing weights - the value cache): per group
// lo = clip * min, hi = clip * max, Delta = (hi - lo) / (2^b - 1), code = clamp(rne((x - lo) / Delta),
// 0, 2^b - 1).  A group is the 16 lanes of a DPP row, 8 values per lane; a wave takes four groups
// per pass.  The extremes cross the 16 lanes with four DPP steps; the codes are taken in fp32 as
// in the rotating kernels (centred on the value that maps to the middle code), and - since
// un-rotated inputs can sit exactly on rounding ties - every value whose fp32 quotient is within 2e-5
// of a tie is retaken with the exact fp64 quotient.
#include "wave_common.h"

namespace rq {
namespace {

// DT: 0 bf16, 1 fp32, 2 fp16.  ALIGNED: 16-byte loads (X 16-byte aligned, ld a multiple of 8 / 4).
template <int DT, bool ALIGNED>
__device__ __forceinline__ void load8(const void* X, int64_t idx, float (&x)[8]) {
    if constexpr (DT == 1) {
        const float* p = static_cast<const float*>(X) + idx;
        if constexpr (ALIGNED) {
            const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
            const u32x4 b = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p) + 1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[i] = __uint_as_float(a[i]);
                x[4 + i] = __uint_as_float(b[i]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = p[i];
        }
    } else {
        const uint16_t* p = static_cast<const uint16_t*>(X) + idx;
        uint32_t w[4];
        if constexpr (ALIGNED) {
            const u32x4 a = load16(p);
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = a[i];
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = (uint32_t)p[2 * i] | ((uint32_t)p[2 * i + 1] << 16);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (DT == 2) {
                x[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)w[i]);
                x[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
            } else {
                x[2 * i] = __uint_as_float(w[i] << 16);
                x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            }
        }
    }
}

template <int BITS, int DT, bool ALIGNED, int U>
__global__ __launch_bounds__(64) void k_plain_asym(const void* X, int64_t n_groups, int gpr, int64_t ld, double clip,
                                                   uint32_t* codes, float* scales, float* mins) {
    constexpr double kL = (double)((1 << BITS) - 1);
    constexpr double kMid = (double)(1 << (BITS - 1)) / kL;
    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    const double c1 = kL / clip;
    const float c1h = (float)c1, c1l = (float)(c1 - (double)c1h);
    // a wave takes U passes of four groups per iteration, all loads issued before the first is used
    for (int64_t g0 = (int64_t)blockIdx.x * (4 * U); g0 < n_groups; g0 += (int64_t)gridDim.x * (4 * U)) {
        float x[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t gi = g0 + u * 4 + g;
            const int64_t gl = gi < n_groups ? gi : n_groups - 1;
            const int64_t row = gpr == 1 ? gl : gl / gpr;
            const int64_t gc = gl - row * gpr;
            load8<DT, ALIGNED>(X, row * ld + gc * 128 + c * 8, x[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t gi = g0 + u * 4 + g;
            const bool live = gi < n_groups;
            float mn = min8(x[u]), mx = max8(x[u]);
            mn = fminf(mn, dpp_f<kDppXor1>(mn));
            mx = fmaxf(mx, dpp_f<kDppXor1>(mx));
            mn = fminf(mn, dpp_f<kDppXor2>(mn));
            mx = fmaxf(mx, dpp_f<kDppXor2>(mx));
            mn = fminf(mn, dpp_f<kDppHalfMirror>(mn));
            mx = fmaxf(mx, dpp_f<kDppHalfMirror>(mx));
            mn = fminf(mn, dpp_f<kDppRor8>(mn));
            mx = fmaxf(mx, dpp_f<kDppRor8>(mx));
            const double lo64 = clip * (double)mn, hi64 = clip * (double)mx;
            // the reported Delta takes a product (one fp64 ulp is far inside its tolerance); the tie
            // decisions below take the quotient itself, since an exact tie turns on the last bit
            const double delta64 = (hi64 - lo64) * (1.0 / kL);
            const double r64 = (double)mx - (double)mn;           // exact
            const float rh = (float)r64, rl = (float)(r64 - (double)rh);
            const bool flat = !(delta64 > 0.0);
            const float s = flat ? 0.0f : div_pair2(c1h, c1l, rh, rl);
            const float cen = (float)(clip * fma(r64, kMid, (double)mn));
            const float bias = flat ? Quant<BITS>::kMagic : Quant<BITS>::kBias;
            uint32_t w = 0;
#pragma unroll
            for (int r = 7; r >= 0; --r) {
                const float dx = x[u][r] - cen;
                float v = fmaf(dx, s, bias);
                const float e = fmaf(dx, s, bias - v);             // t - round(t)
                v = __builtin_amdgcn_fmed3f(v, Quant<BITS>::kLo, Quant<BITS>::kHi);
                // within 2e-5 of a rounding tie (five times the worst fp32 error of t, 4e-6; four values in
                // a hundred thousand): the exact fp64 quotient decides, for this value only
                if (__builtin_fabsf(e) > 0.49998f && !flat)
                    v = Quant<BITS>::kMagic +
                        (float)fmin(fmax(rint(((double)x[u][r] - lo64) / ((hi64 - lo64) / kL)), 0.0), kL);
                w = (w << BITS) + __float_as_uint(v);
            }
            w -= Quant<BITS>::csum();
            if (BITS == 4) {
                if (live) store_codes(codes + gi * 16 + c, w);
            } else {
                const int qpos = c & 3;
                const uint32_t dw = merge24<false>(w, qpos);
                if (live && qpos < 3) store_codes(codes + gi * 12 + (c >> 2) * 3 + qpos, dw);
            }
            if (live && c == 0) {
                scales[gi] = (float)delta64;
                mins[gi] = (float)lo64;
            }
        }
    }
}

template <int DT>
void launch_dt(bool aligned, int bits, unsigned grid, hipStream_t s, const void* X, int64_t n_groups, int gpr,
               int64_t ld, double clip, uint32_t* codes, float* scales, float* mins) {
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, X, n_groups, gpr, ld, clip, codes, scales, mins); };
    if (aligned) {
        if (bits == 4) go(k_plain_asym<4, DT, true, 4>); else go(k_plain_asym<3, DT, true, 4>);
    } else {
        if (bits == 4) go(k_plain_asym<4, DT, false, 4>); else go(k_plain_asym<3, DT, false, 4>);
    }
}

}  // namespace

int plain_quantize_asym(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                        uint32_t* codes, float* scales, float* mins, hipStream_t s) {
    const int gpr = d / RQ_GROUP;
    const int64_t n_groups = rows * gpr;
    const int64_t passes = (n_groups + 15) / 16;          // 4 groups x 4 passes per wave iteration
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(passes < cap ? passes : cap);
    const int esz = dtype == RQ_F32 ? 4 : 2;
    const bool aligned = (reinterpret_cast<uintptr_t>(X) & 15) == 0 && (ld * esz) % 16 == 0;
    if (dtype == RQ_BF16) launch_dt<0>(aligned, bits, grid, s, X, n_groups, gpr, ld, (double)clip, codes, scales, mins);
    else if (dtype == RQ_F32) launch_dt<1>(aligned, bits, grid, s, X, n_groups, gpr, ld, (double)clip, codes, scales, mins);
    else launch_dt<2>(aligned, bits, grid, s, X, n_groups, gpr, ld, (double)clip, codes, scales, mins);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace rq
