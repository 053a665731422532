// Rotation-free quantizers for short groups of values (head rows).
// First the asymmetric quantizer in groups of 128 values (section 5.1, the KV-cache setting, for
// a tensor whose rotation is fused into the producing weights - the value cache): per group
// lo = clip * min, hi = clip * max, Delta = (hi - lo) / (2^b - 1), code = clamp(rne((x - lo) / Delta),
// 0, 2^b - 1).  A group is the 16 lanes of a DPP row, 8 values per lane; a wave takes four groups
// per pass.  The extremes cross the 16 lanes with four DPP steps; the codes are taken in fp32 as
// in the rotating kernels (centred on the value that maps to the middle code), and - since
// un-rotated inputs can sit exactly on rounding ties - every value whose fp32 quotient is within 2e-5
// of a tie (wider for a group that lies far from zero, where fp32 places the centre less well) is
// retaken with the exact fp64 quotient.
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

// Minimum of mn and maximum of mx over the 16 lanes of a DPP row, every lane ending with both: four
// butterfly steps, each one instruction with a DPP operand (assembly: the compiler does not fold a DPP
// operand into a float min / max, and first passes each operand through a canonicalizing max).  The
// s_nop keep two wait states between a vector write of a register and a DPP read of it.
__device__ __forceinline__ void row_min_max(float& mn, float& mx) {
    asm("s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_min_f32_dpp %0, %0, %0 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(mn), "+v"(mx));
}

// max |y_k| of eight floats as three-operand instructions with magnitude operands
__device__ __forceinline__ float absmax8(const float (&y)[8]) {
    float m;
    asm("v_max3_f32 %0, |%1|, |%2|, |%3|\n\t"
        "v_max3_f32 %0, %0, |%4|, |%5|\n\t"
        "v_max3_f32 %0, %0, |%6|, |%7|\n\t"
        "v_max_f32 %0, %0, |%8|"
        : "=&v"(m)
        : "v"(y[0]), "v"(y[1]), "v"(y[2]), "v"(y[3]), "v"(y[4]), "v"(y[5]), "v"(y[6]), "v"(y[7]));
    return m;
}

template <int BITS, int DT, bool ALIGNED, int U>
__global__ __launch_bounds__(64) void k_plain_asym(const void* X, int64_t n_groups, int gpr, int gpr_shift, uint32_t gpr_magic, int64_t ld, double clip,
                                                   uint32_t* codes, float* scales, float* mins) {
    constexpr double kL = (double)((1 << BITS) - 1);
    constexpr double kMid = (double)(1 << (BITS - 1)) / kL;     // centre of the code range
    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    constexpr float kMidF = (float)kMid;
    const float c1f = (float)(kL / clip), clipf = (float)clip;
    // a wave takes U passes of four groups per iteration, all loads issued before the first is used
    for (int64_t g0 = (int64_t)blockIdx.x * (4 * U); g0 < n_groups; g0 += (int64_t)gridDim.x * (4 * U)) {
        float x[U][8];
        // uniform over the wave, so scalar work - but a 64-bit scalar division is a hundred instructions:
        // a shift where gpr is a power of two (the usual widths), else a 32-bit division if that will do
        int64_t row0;
        if (gpr_shift >= 0) row0 = g0 >> gpr_shift;
        else if (n_groups <= 0xffffffffll) row0 = (uint32_t)g0 / (uint32_t)gpr;
        else row0 = g0 / gpr;
        const uint32_t rem0 = (uint32_t)(g0 - row0 * gpr);
        // outputs of the iteration: a base in scalar registers plus per-lane offsets; lane c of a group
        // keeps the parameters of pass c, so that the iteration's U * 4 scales and minima leave in one store each
        uint32_t* const cbase = codes + g0 * (4 * BITS);
        const uint32_t code_off = (uint32_t)(g * (4 * BITS) + (BITS == 4 ? c : (c >> 2) * 3 + (c & 3))) * 4u;
        uint32_t* const out0 = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(cbase) + code_off);
        float keep_d = 0.0f, keep_m = 0.0f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t gi = g0 + u * 4 + g;
            const int64_t gl = gi < n_groups ? gi : n_groups - 1;
            // (row, group of the row) from the iteration's uniform split plus a small offset, whose
            // quotient by gpr is a multiply-high with ceil(2^32 / gpr): exact while offset * gpr < 2^32
            const uint32_t off = rem0 + (uint32_t)(gl - g0);
            const uint32_t k = gpr == 1 ? off : __umulhi(off, gpr_magic);
            const int64_t row = row0 + k;
            const uint32_t gc = off - k * (uint32_t)gpr;
            load8<DT, ALIGNED>(X, row * ld + (int64_t)gc * 128 + c * 8, x[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t gi = g0 + u * 4 + g;
            const bool live = gi < n_groups;
            float mn = min8(x[u]), mx = max8(x[u]);
            row_min_max(mn, mx);
            // Group parameters in fp32.  What they cost the pre-round value t in accuracy: the range r
            // and the multiplier s (reciprocal plus one Newton step) about 3e-7 relative, |t - mid| <= 8;
            // the centre about 2.5 ulp, which in units of t is 3e-7 |cen| s - small for a group that
            // straddles zero, unbounded for a narrow group far from it.  Both go into the tie window, so
            // a group whose offset swamps its range is simply taken in fp64 throughout.
            const float r = mx - mn;
            const bool flat = !(r > 0.0f);
            float q = __builtin_amdgcn_rcpf(r);
            q = fmaf(fmaf(-r, q, 1.0f), q, q);
            const float s = flat ? 0.0f : c1f * q;
            const float cen = clipf * fmaf(r, kMidF, mn);
            // (a range whose reciprocal is subnormal - the reciprocal instruction returns zero for it -
            // or so small that s overflows leaves no window at all)
            const float thr = (r < 4e37f && s < 1e30f) ? fmaf(-3e-7f * __builtin_fabsf(cen), s, 0.49998f) : -1.0f;
            const float bias = flat ? Quant<BITS>::kMagic : Quant<BITS>::kBias;
            float v[8], e[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float dx = x[u][k] - cen;
                v[k] = fmaf(dx, s, bias);
                e[k] = fmaf(dx, s, bias - v[k]);                   // t - round(t)
            }
            // near a rounding tie: the definition itself, in fp64 and with its two divisions (an exact tie
            // turns on their last bit), for that value only; one test per lane and pass guards the lot
            const float emax = absmax8(e);
            if (!(emax <= thr) && !flat) {
                float mn_here = mn;
                asm volatile("" : "+v"(mn_here));                  // keeps the fp64 work inside the branch
                const double lo64 = clip * (double)mn_here, hi64 = clip * (double)mx;
                const double delta64 = (hi64 - lo64) / kL;
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (!(__builtin_fabsf(e[k]) <= thr))
                        v[k] = Quant<BITS>::kMagic + (float)fmin(fmax(rint(((double)x[u][k] - lo64) / delta64), 0.0), kL);
            }
            uint32_t w = 0;
#pragma unroll
            for (int k = 7; k >= 0; --k)
                w = (w << BITS) + __float_as_uint(__builtin_amdgcn_fmed3f(v[k], Quant<BITS>::kLo, Quant<BITS>::kHi));
            w -= Quant<BITS>::csum();
            if (BITS == 4) {
                if (live) store_codes(out0 + u * (16 * BITS), w);
            } else {
                const int qpos = c & 3;
                const uint32_t dw = merge24<false>(w, qpos);
                if (live && qpos < 3) store_codes(out0 + u * (16 * BITS), dw);
            }
            float delta = clipf * r * (float)(1.0 / kL);            // each factor good to 6e-8
            if (!(r < 3e38f)) {                                     // max - min beyond fp32
                float mx_here = mx;
                asm volatile("" : "+v"(mx_here));
                delta = (float)((clip * (double)mx_here - clip * (double)mn) * (1.0 / kL));
            }
            keep_d = c == u ? delta : keep_d;
            keep_m = c == u ? clipf * mn : keep_m;
        }
        const int64_t gs = g0 + c * 4 + g;                          // lane c < U: group of pass c
        if (c < U && gs < n_groups) {
            scales[gs] = keep_d;
            mins[gs] = keep_m;
        }
    }
}

// Per-token symmetric quantizer (section 2.1) for short rows, d <= 8 LPR <= 512 - head rows that arrive
// already rotated: LPR = 16, 32 or 64 lanes hold a row, 8 values each, so a wave takes 4, 2 or 1 rows
// per pass and U passes per iteration.  Same scheme as above without the offset: absmax over the row's
// lanes (bit patterns of non-negative floats order like unsigned integers), s = (2^b - 1) / (clip amax)
// in fp32, codes by one fused multiply-add, values within 2e-5 of a tie retaken from the exact fp64
// quotient x / Delta.
template <int BITS, int DT, int LPR, int U>
__global__ __launch_bounds__(64) void k_plain_short(const void* X, int64_t rows, int d, int64_t ld, double clip,
                                                    uint32_t* codes, float* scales) {
    constexpr double kL = (double)((1 << BITS) - 1);
    constexpr int RPP = 64 / LPR;                                 // rows per pass
    constexpr float kQmin = -(float)(1 << (BITS - 1)), kQmax = (float)((1 << (BITS - 1)) - 1);
    const int lane = threadIdx.x;
    const int sr = lane / LPR, c = lane % LPR;
    const bool has = c * 8 < d;                                   // d is a multiple of 32: whole quads of lanes
    const int row_dwords = d * BITS / 32;
    const float c1f = (float)(kL / clip), clipf = (float)clip;
    for (int64_t r0 = (int64_t)blockIdx.x * (RPP * U); r0 < rows; r0 += (int64_t)gridDim.x * (RPP * U)) {
        float x[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = r0 + u * RPP + sr;
            const int64_t rl = row < rows ? row : rows - 1;
            if (has) load8<DT, true>(X, rl * ld + c * 8, x[u]);
            else
#pragma unroll
                for (int k = 0; k < 8; ++k) x[u][k] = 0.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = r0 + u * RPP + sr;
            const bool live = row < rows && has;
            uint32_t mi = __float_as_uint(absmax8(x[u]));
            mi = max(mi, dpp_u<kDppXor1>(mi));
            mi = max(mi, dpp_u<kDppXor2>(mi));
            mi = max(mi, dpp_u<kDppHalfMirror>(mi));
            mi = max(mi, dpp_u<kDppRor8>(mi));
            if constexpr (LPR >= 32) {                            // DPP rows 0 | 1 and 2 | 3
                const auto a = __builtin_amdgcn_permlane16_swap(mi, mi, false, false);
                mi = max((uint32_t)a[0], (uint32_t)a[1]);
            }
            if constexpr (LPR == 64) {
                const auto b = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);
                mi = max((uint32_t)b[0], (uint32_t)b[1]);
            }
            const float m = __uint_as_float(mi);
            const bool flat = !(m > 0.0f);
            float q = __builtin_amdgcn_rcpf(m);
            q = fmaf(fmaf(-m, q, 1.0f), q, q);
            const float s = flat ? 0.0f : c1f * q;
            // (no window where the reciprocal of amax is subnormal or s overflows: fp64 throughout)
            const float thr = (m < 4e37f && s < 1e30f) ? 0.49998f : -1.0f;
            float v[8], e[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                v[k] = fmaf(x[u][k], s, Quant<BITS>::kBias);
                e[k] = fmaf(x[u][k], s, Quant<BITS>::kBias - v[k]);     // t - round(t)
            }
            const float emax = absmax8(e);
            if (!(emax <= thr) && !flat) {
                float m_here = m;
                asm volatile("" : "+v"(m_here));                  // keeps the fp64 work inside the branch
                const double delta64 = clip * (double)m_here / kL;
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (!(__builtin_fabsf(e[k]) <= thr))
                        v[k] = Quant<BITS>::kBias + fminf(fmaxf((float)rint((double)x[u][k] / delta64), kQmin), kQmax);
            }
            uint32_t w = 0;
#pragma unroll
            for (int k = 7; k >= 0; --k)
                w = (w << BITS) + __float_as_uint(__builtin_amdgcn_fmed3f(v[k], Quant<BITS>::kLo, Quant<BITS>::kHi));
            w = (w - Quant<BITS>::csum()) ^ Quant<BITS>::msb();
            uint32_t* out = codes + row * (int64_t)row_dwords;
            if (BITS == 4) {
                if (live) store_codes(out + c, w);
            } else {
                const int qpos = c & 3;
                const uint32_t dw = merge24<false>(w, qpos);
                if (live && qpos < 3) store_codes(out + (c >> 2) * 3 + qpos, dw);
            }
            if (live && c == 0) scales[row] = clipf * m * (float)(1.0 / kL);
        }
    }
}

template <int DT, int LPR>
void launch_short(int bits, hipStream_t s, const void* X, int64_t rows, int d, int64_t ld, double clip,
                  uint32_t* codes, float* scales) {
    constexpr int U = 4;
    const int64_t iters = (rows + (64 / LPR) * U - 1) / ((64 / LPR) * U);
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(iters < cap ? iters : cap);
    if (bits == 4) hipLaunchKernelGGL((k_plain_short<4, DT, LPR, U>), dim3(grid), dim3(64), 0, s, X, rows, d, ld, clip, codes, scales);
    else hipLaunchKernelGGL((k_plain_short<3, DT, LPR, U>), dim3(grid), dim3(64), 0, s, X, rows, d, ld, clip, codes, scales);
}

template <int DT>
void launch_short_dt(int bits, hipStream_t s, const void* X, int64_t rows, int d, int64_t ld, double clip,
                     uint32_t* codes, float* scales) {
    if (d <= 128) launch_short<DT, 16>(bits, s, X, rows, d, ld, clip, codes, scales);
    else if (d <= 256) launch_short<DT, 32>(bits, s, X, rows, d, ld, clip, codes, scales);
    else launch_short<DT, 64>(bits, s, X, rows, d, ld, clip, codes, scales);
}

template <int DT>
void launch_dt(bool aligned, int bits, unsigned grid, hipStream_t s, const void* X, int64_t n_groups, int gpr,
               int64_t ld, double clip, uint32_t* codes, float* scales, float* mins) {
    const int gpr_shift = (gpr & (gpr - 1)) == 0 ? __builtin_ctz((unsigned)gpr) : -1;
    const uint32_t gpr_magic = (uint32_t)((((uint64_t)1 << 32) + gpr - 1) / gpr);   // gpr >= 2 where it is used
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, X, n_groups, gpr, gpr_shift, gpr_magic, ld, clip, codes, scales, mins); };
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

bool plain_short_supports(const void* X, int dtype, int d, int64_t ld) {
    const int esz = dtype == RQ_F32 ? 4 : 2;
    return d <= 512 && d % 32 == 0 && (reinterpret_cast<uintptr_t>(X) & 15) == 0 && (ld * esz) % 16 == 0;
}

int plain_short_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                         uint32_t* codes, float* scales, hipStream_t s) {
    if (dtype == RQ_BF16) launch_short_dt<0>(bits, s, X, rows, d, ld, (double)clip, codes, scales);
    else if (dtype == RQ_F32) launch_short_dt<1>(bits, s, X, rows, d, ld, (double)clip, codes, scales);
    else launch_short_dt<2>(bits, s, X, rows, d, ld, (double)clip, codes, scales);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace rq
