// Device helpers shared by the wave-level kernels: DPP permutations, the fused cross-lane
// butterfly stages, chunk loads, and the launch-argument block.
#pragma once
#include "rotq_internal.h"

namespace rq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// One matrix-core step D = A * B + C with 16-bit operands held as four dwords: bf16, or IEEE fp16
// when F16 (the +-1 operand tile is then encoded in fp16 as well).  Products with +-1 are exact
// in both formats; accumulation is fp32.
template <bool F16>
__device__ __forceinline__ float __attribute__((ext_vector_type(4)))
mfma_pm1(const u32x4& a, const u32x4& b, const float __attribute__((ext_vector_type(4))) & c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

constexpr int kDppXor1 = 0xB1;         // quad_perm:[1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // row_half_mirror: lane i <-> 7 - i
constexpr int kDppRor8 = 0x128;        // row_ror:8: lane i <-> i ^ 8
constexpr int kDppNext = 0xF9;         // quad_perm:[1,2,3,3]: value of the next lane of the quad
constexpr int kDppPrev = 0x90;         // quad_perm:[0,0,1,2]: value of the previous lane

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

// One cross-lane butterfly stage in place: partner + (upper lane ? -self : self), i.e. a + b on
// the lower lane of a pair and a - b on the upper one (one sign flip plus one DPP add).
template <int CTRL>
__device__ __forceinline__ void lane_stage(f32x4& v, uint32_t signbit) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float x = v[i];   // scalar copy: bit-casting a vector element in place is not reliable
        const float self = __uint_as_float(__float_as_uint(x) ^ signbit);
        v[i] = dpp_f<CTRL>(x) + self;
    }
}

// The four cross-lane stages (xor-1, xor-2, half mirror, xor-8) on four independent values, one
// v_fmac_f32 with a DPP-permuted operand per value and stage: x <- x + sign * partner(x), sign
// = -1 on the upper lane of a pair.  The upper lane thus receives b - a instead of a - b; these
// negations commute with all later stages and are undone once, in the sign of the lane's
// quantization multiplier.  (The compiler does not fold a DPP operand into an fma, hence the
// assembly.)  A DPP read needs two wait states after the VALU write of its source: the leading
// s_nop covers the producer of the inputs, and inside the block three instructions separate a
// value's consecutive stages.
__device__ __forceinline__ void lane_stages_fused(f32x4& v, float s0, float s1, float s2, float s3) {
    float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %4 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %4 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %4 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %4 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %5 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %5 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %5 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %5 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %6 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %6 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %6 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %6 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %7 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %7 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %7 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %7 row_ror:8 row_mask:0xf bank_mask:0xf"
        : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
        : "v"(s0), "v"(s1), "v"(s2), "v"(s3));
    v[0] = x0; v[1] = x1; v[2] = x2; v[3] = x3;
}

// Stages 2 .. CB (xor-2, half mirror, xor-8) fused as above, for values that come straight from
// the matrix cores: stage 1 is then taken with lane_stage, whose instructions the compiler sees
// and separates from the matrix-core write by the required wait states (it does not look inside
// an assembly block).
__device__ __forceinline__ void lane_stages_tail_1(f32x4& v, float s1) {
    float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
        : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
        : "v"(s1));
    v[0] = x0; v[1] = x1; v[2] = x2; v[3] = x3;
}
__device__ __forceinline__ void lane_stages_tail_2(f32x4& v, float s1, float s2) {
    float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %5 row_half_mirror row_mask:0xf bank_mask:0xf"
        : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
        : "v"(s1), "v"(s2));
    v[0] = x0; v[1] = x1; v[2] = x2; v[3] = x3;
}
__device__ __forceinline__ void lane_stages_tail_3(f32x4& v, float s1, float s2, float s3) {
    float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %6 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %6 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %6 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %3, %6 row_ror:8 row_mask:0xf bank_mask:0xf"
        : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
        : "v"(s1), "v"(s2), "v"(s3));
    v[0] = x0; v[1] = x1; v[2] = x2; v[3] = x3;
}

template <int CB>
__device__ __forceinline__ void lane_stages_tail(f32x4& v, const float (&sf)[4]) {
    if constexpr (CB == 2) lane_stages_tail_1(v, sf[1]);
    else if constexpr (CB == 3) lane_stages_tail_2(v, sf[1], sf[2]);
    else lane_stages_tail_3(v, sf[1], sf[2], sf[3]);
}

// All CB stages for the four results of one matrix-core instruction, in the fused convention
// throughout (so the lane sign is the parity of all CB bits).  Only the first element's first
// stage is code the compiler sees: it puts the wait states a matrix-core write needs in front
// of that read, all four result registers are written by then, and the assembly block - which
// takes that element as an operand and so cannot move ahead of it - may read the other three.
template <int CB>
__device__ __forceinline__ void lane_stages_mfma(f32x4& v, const float (&sf)[4]) {
    float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3];
    x0 = fmaf(dpp_f<kDppXor1>(x0), sf[0], x0);
#define RQ_ST1(r) "v_fmac_f32_dpp " r ", " r ", %4 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
#define RQ_ST2(r) "v_fmac_f32_dpp " r ", " r ", %5 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
#define RQ_ST3(r) "v_fmac_f32_dpp " r ", " r ", %6 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
#define RQ_ST4(r) "v_fmac_f32_dpp " r ", " r ", %7 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
    if constexpr (CB == 2)
        asm("s_nop 1\n\t" RQ_ST1("%1") RQ_ST1("%2") RQ_ST1("%3")
            RQ_ST2("%0") RQ_ST2("%1") RQ_ST2("%2") RQ_ST2("%3")
            : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
            : "v"(sf[0]), "v"(sf[1]), "v"(sf[2]), "v"(sf[3]));
    else if constexpr (CB == 3)
        asm("s_nop 1\n\t" RQ_ST1("%1") RQ_ST1("%2") RQ_ST1("%3")
            RQ_ST2("%0") RQ_ST2("%1") RQ_ST2("%2") RQ_ST2("%3")
            RQ_ST3("%0") RQ_ST3("%1") RQ_ST3("%2") RQ_ST3("%3")
            : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
            : "v"(sf[0]), "v"(sf[1]), "v"(sf[2]), "v"(sf[3]));
    else
        asm("s_nop 1\n\t" RQ_ST1("%1") RQ_ST1("%2") RQ_ST1("%3")
            RQ_ST2("%0") RQ_ST2("%1") RQ_ST2("%2") RQ_ST2("%3")
            RQ_ST3("%0") RQ_ST3("%1") RQ_ST3("%2") RQ_ST3("%3")
            RQ_ST4("%0") RQ_ST4("%1") RQ_ST4("%2") RQ_ST4("%3")
            : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3)
            : "v"(sf[0]), "v"(sf[1]), "v"(sf[2]), "v"(sf[3]));
#undef RQ_ST1
#undef RQ_ST2
#undef RQ_ST3
#undef RQ_ST4
    v[0] = x0; v[1] = x1; v[2] = x2; v[3] = x3;
}

// The same on one, two or three values; with fewer than three values in flight an s_nop keeps
// two wait states between a value's consecutive stages.
__device__ __forceinline__ void lane_stages_fused1(float& x0, float s0, float s1, float s2, float s3) {
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %2 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %3 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %4 row_ror:8 row_mask:0xf bank_mask:0xf"
        : "+v"(x0)
        : "v"(s0), "v"(s1), "v"(s2), "v"(s3));
}
__device__ __forceinline__ void lane_stages_fused2(float& x0, float& x1, float s0, float s1, float s2, float s3) {
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %2 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %2 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_fmac_f32_dpp %0, %0, %3 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %3 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_fmac_f32_dpp %0, %0, %4 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %4 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_fmac_f32_dpp %0, %0, %5 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %5 row_ror:8 row_mask:0xf bank_mask:0xf"
        : "+v"(x0), "+v"(x1)
        : "v"(s0), "v"(s1), "v"(s2), "v"(s3));
}
__device__ __forceinline__ void lane_stages_fused3(float& x0, float& x1, float& x2, float s0, float s1, float s2, float s3) {
    asm("s_nop 1\n\t"
        "v_fmac_f32_dpp %0, %0, %3 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %3 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %3 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %5 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %0, %6 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %1, %6 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %2, %6 row_ror:8 row_mask:0xf bank_mask:0xf"
        : "+v"(x0), "+v"(x1), "+v"(x2)
        : "v"(s0), "v"(s1), "v"(s2), "v"(s3));
}

__device__ __forceinline__ float absmax4(float m, const f32x4& v) {
    m = __builtin_fmaxf(__builtin_fmaxf(m, __builtin_fabsf(v[0])), __builtin_fabsf(v[1]));
    return __builtin_fmaxf(__builtin_fmaxf(m, __builtin_fabsf(v[2])), __builtin_fabsf(v[3]));
}

// A row of width d (a multiple of 8) as a raw buffer resource: loads beyond the row's d * 2
// bytes return zero in hardware, which is the zero padding of section 4.2 with no compare or
// select in the instruction stream.  `row` must be uniform across the wave.
struct RowView {
    __amdgpu_buffer_rsrc_t rs;
};
__device__ __forceinline__ RowView row_view(const uint16_t* row, int d) {
    return RowView{__builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(row), 0, d * 2, 0x00020000)};
}
// 16-byte chunk starting at element e0 (a multiple of 8): whole chunks only, zero beyond d.
// Streamed once: non-temporal, so the row does not displace anything in the caches.
__device__ __forceinline__ u32x4 load_chunk(const RowView& v, int e0) {
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(v.rs, e0 * 2, 0, 2));
}

struct WaveArgs {
    const uint16_t* X;
    int64_t rows;
    int d;
    int64_t ld;
    const u32x4* tiles;   // matrix-core operand of the 32x32 +-1 block: [2][64] x 16 bytes
    uint32_t* codes;
    float* scales;
    double c1;            // (2^b - 1) / clip
    double c2;            // clip / (sqrt(n) (2^b - 1))
    // asymmetric group variant only
    float* mins = nullptr;
    double clip = 0.0;
    double c3 = 0.0;      // clip / sqrt(n)
    bool f16 = false;     // X holds IEEE fp16 instead of bf16 (tiles must be the fp16 table then)
};


// Quantizer constants for b-bit codes (section 2.1 with the clip ratio of section 3.1).
// u = fma(y, s, kBias) rounds y*s + 2^(b-1) to the nearest-even integer on the fp32 lattice
// above 1.5 * 2^23; v_med3 clamps it to [kLo, kHi]; the code (offset binary) is the low
// mantissa bits.  Eight codes are chained with shift-adds, the accumulated exponent bits
// (kCsum) are subtracted once and one xor (kMsb) turns offset binary into two's complement.
template <int BITS>
struct Quant {
    static constexpr float kMagic = 12582912.0f;   // 1.5 * 2^23
    static constexpr float kLo = kMagic, kHi = kMagic + (float)((1 << BITS) - 1);
    static constexpr float kBias = kMagic + (float)(1 << (BITS - 1));
    static constexpr uint32_t csum() {
        uint32_t c = 0;
        for (int r = 0; r < 8; ++r) c += 0x4B400000u << (BITS * r);
        return c;
    }
    static constexpr uint32_t msb() {
        uint32_t m = 0;
        for (int r = 0; r < 8; ++r) m |= 1u << (BITS * r + BITS - 1);
        return m;
    }
    // packs codes of y0..y7 (y0 in the low bits) into 8*BITS bits
    static __device__ __forceinline__ uint32_t pack8(float y0, float y1, float y2, float y3, float y4,
                                                     float y5, float y6, float y7, float s) {
        const float y[8] = {y0, y1, y2, y3, y4, y5, y6, y7};
        uint32_t w = 0;
#pragma unroll
        for (int r = 7; r >= 0; --r) {
            float u = fmaf(y[r], s, kBias);
            u = __builtin_amdgcn_fmed3f(u, kLo, kHi);
            w = (w << BITS) + __float_as_uint(u);
        }
        return (w - csum()) ^ msb();
    }
    // Unsigned codes 0 .. 2^b - 1 of (y - cen) * s + bias - kMagic: the asymmetric group
    // quantizer, centred on the value `cen` that maps to the middle code so that the fp32
    // products stay as small as in the symmetric case.
    static __device__ __forceinline__ uint32_t pack8u(const float (&y)[8], float cen, float s, float bias) {
        uint32_t w = 0;
#pragma unroll
        for (int r = 7; r >= 0; --r) {
            float u = fmaf(y[r] - cen, s, bias);
            u = __builtin_amdgcn_fmed3f(u, kLo, kHi);
            w = (w << BITS) + __float_as_uint(u);
        }
        return w - csum();
    }
};

// b = 3: a lane's 24 bits and those of the lane holding the next 8 columns (lane + 1, or
// lane - 1 in mirrored quads) make the dword for quad position qpos (0..2).
template <bool MIRROR>
__device__ __forceinline__ uint32_t merge24(uint32_t w, int qpos) {
    uint32_t nxt;
    if constexpr (MIRROR) {
        nxt = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, kDppNext, 0xf, 0x5, true);
        nxt = (uint32_t)__builtin_amdgcn_update_dpp((int)nxt, (int)w, kDppPrev, 0xf, 0xa, false);
    } else {
        nxt = dpp_u<kDppNext>(w);
    }
    return (w >> (8 * qpos)) | (nxt << (24 - 8 * qpos));
}

// b = 3 output path.  A lane holds 24 bits per group of 8 columns, which is not a whole dword;
// the row's packed bytes are therefore assembled in LDS (three byte writes per group, no
// cross-lane merging, no per-group predicates) and then copied to memory as 16-byte units by
// all lanes.  `stage` is private to the wave's workgroup and 16-byte aligned.
__device__ __forceinline__ void stage24(uint8_t* stage, int group, uint32_t w) {
    uint8_t* p = stage + group * 3;
    p[0] = (uint8_t)w;
    p[1] = (uint8_t)(w >> 8);
    p[2] = (uint8_t)(w >> 16);
}

template <int MAX_UNITS>
__device__ __forceinline__ void copy_out16(const uint8_t* stage, uint32_t* out, int units, int lane) {
#pragma unroll
    for (int k = 0; k * 64 < MAX_UNITS; ++k) {
        const int idx = k * 64 + lane;
        if (idx < units)
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(stage + idx * 16),
                                        reinterpret_cast<u32x4*>(out) + idx);
    }
}

// Packed codes are written once and not read back by this kernel: non-temporal store.
__device__ __forceinline__ void store_codes(uint32_t* p, uint32_t v) { __builtin_nontemporal_store(v, p); }

// The four fused cross-lane stages on N (1..4) consecutive values.
template <int N>
__device__ __forceinline__ void fused_group(float* v, const float (&sf)[4]) {
    if constexpr (N == 4) {
        f32x4 q = {v[0], v[1], v[2], v[3]};
        lane_stages_fused(q, sf[0], sf[1], sf[2], sf[3]);
        v[0] = q[0]; v[1] = q[1]; v[2] = q[2]; v[3] = q[3];
    } else if constexpr (N == 3) {
        lane_stages_fused3(v[0], v[1], v[2], sf[0], sf[1], sf[2], sf[3]);
    } else if constexpr (N == 2) {
        lane_stages_fused2(v[0], v[1], sf[0], sf[1], sf[2], sf[3]);
    } else {
        lane_stages_fused1(v[0], sf[0], sf[1], sf[2], sf[3]);
    }
}

// Max over the four DPP rows of a wave (lanes l, l ^ 16, l ^ 32, l ^ 48) with the row-swap
// instructions: v_permlane16_swap(a, b) returns rows [a0 b0 a2 b2] and [a1 b1 a3 b3],
// v_permlane32_swap(a, b) returns [a0 a1 b0 b1] and [a2 a3 b2 b3]; no LDS traffic.
__device__ __forceinline__ uint32_t rows_max_u32(uint32_t m) {
    const auto a = __builtin_amdgcn_permlane16_swap(m, m, false, false);
    m = max((uint32_t)a[0], (uint32_t)a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(m, m, false, false);
    return max((uint32_t)b[0], (uint32_t)b[1]);
}

// Sum over the four DPP rows of a wave with the same two row swaps: every lane ends with the total.
__device__ __forceinline__ float rows_sum(float v) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float((uint32_t)a[0]) + __uint_as_float((uint32_t)a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float((uint32_t)b[0]) + __uint_as_float((uint32_t)b[1]);
}

// Max of a non-negative float over lanes: non-negative floats order like their bit patterns,
// so the reduction runs on unsigned integers (one DPP-fused v_max_u32 per step).  ROW_BITS of
// the four DPP row patterns are used (lanes that share a row differ in those bits), then the two
// cross-row steps.
template <int ROW_BITS = 4>
__device__ __forceinline__ float wave_absmax(float mf) {
    uint32_t m = __float_as_uint(mf);
    m = max(m, dpp_u<kDppXor1>(m));
    m = max(m, dpp_u<kDppXor2>(m));
    if (ROW_BITS >= 3) m = max(m, dpp_u<kDppHalfMirror>(m));
    if (ROW_BITS >= 4) m = max(m, dpp_u<kDppRor8>(m));
    return __uint_as_float(rows_max_u32(m));
}

// Min / max of eight floats as three-operand instructions.  Written in assembly because the
// values come out of an assembly block: the compiler would first pass each of them through a
// canonicalizing v_max_f32 x, x, which costs as much as the reduction itself.
__device__ __forceinline__ float max8(const float (&y)[8]) {
    float m;
    asm("v_max3_f32 %0, %1, %2, %3\n\t"
        "v_max3_f32 %0, %0, %4, %5\n\t"
        "v_max3_f32 %0, %0, %6, %7\n\t"
        "v_max_f32 %0, %0, %8"
        : "=&v"(m)
        : "v"(y[0]), "v"(y[1]), "v"(y[2]), "v"(y[3]), "v"(y[4]), "v"(y[5]), "v"(y[6]), "v"(y[7]));
    return m;
}
__device__ __forceinline__ float min8(const float (&y)[8]) {
    float m;
    asm("v_min3_f32 %0, %1, %2, %3\n\t"
        "v_min3_f32 %0, %0, %4, %5\n\t"
        "v_min3_f32 %0, %0, %6, %7\n\t"
        "v_min_f32 %0, %0, %8"
        : "=&v"(m)
        : "v"(y[0]), "v"(y[1]), "v"(y[2]), "v"(y[3]), "v"(y[4]), "v"(y[5]), "v"(y[6]), "v"(y[7]));
    return m;
}

// Max of two floats at once (mx and nm = -min) over the 4 lanes of a quad and the four DPP rows:
// the lanes that hold one row of 128 values.  The quad steps are DPP-fused maxima (assembly: the
// compiler does not fold a DPP operand into a float max); the row steps carry mx in rows 0 / 2
// and nm in rows 1 / 3, so that three row swaps and two maxima serve both values.
__device__ __forceinline__ void quad_rows_max_pair(float& mx, float& nm) {
    asm("s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 3"
        : "+v"(mx), "+v"(nm));
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(mx), __float_as_uint(nm), false, false);
    float x = __builtin_fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __builtin_fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
    const auto c = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    mx = __uint_as_float(c[0]);
    nm = __uint_as_float(c[1]);
}

// c / m for m > 0 with c = ch + cl (float pair): reciprocal, one Newton step, one correction of
// the quotient, then the low part; about half an ulp.  Used where a full IEEE division per
// row would be a visible cost (short rows).
__device__ __forceinline__ float div_pair(float ch, float cl, float m) {
    float r = __builtin_amdgcn_rcpf(m);
    r = fmaf(fmaf(-m, r, 1.0f), r, r);
    float q = ch * r;
    q = fmaf(fmaf(-q, m, ch), r, q);
    return fmaf(cl, r, q);
}

// (ch + cl) / (mh + ml), mh > 0, |ml| <= ulp(mh) / 2: as div_pair with the divisor's low part
// folded into the last correction.
__device__ __forceinline__ float div_pair2(float ch, float cl, float mh, float ml) {
    float r = __builtin_amdgcn_rcpf(mh);
    r = fmaf(fmaf(-mh, r, 1.0f), r, r);
    float q = ch * r;
    q = fmaf(fmaf(-q, mh, ch), r, q);
    return fmaf(fmaf(-q, ml, cl), r, q);
}

// 16-byte non-temporal load of a whole chunk (no bounds handling).
__device__ __forceinline__ u32x4 load16(const uint16_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// Eight consecutive results of a lane (carrying the lane's sign in `k`) to columns col .. col + 7.
// OUT: 0 bf16, 1 fp32, 2 fp16 (round to nearest even).
template <int OUT>
__device__ __forceinline__ void store8(void* Y, int64_t idx, const float (&v)[8], float k, float add0 = 0.0f) {
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = v[i] * k;
    o[0] += add0;
    if constexpr (OUT == 1) {
        u32x4* p = reinterpret_cast<u32x4*>(static_cast<float*>(Y) + idx);
        p[0] = u32x4{__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3])};
        p[1] = u32x4{__float_as_uint(o[4]), __float_as_uint(o[5]), __float_as_uint(o[6]), __float_as_uint(o[7])};
    } else {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t lo, hi;
            if constexpr (OUT == 0) {
                const uint32_t a = __float_as_uint(o[2 * i]), b = __float_as_uint(o[2 * i + 1]);
                lo = (a + 0x7fffu + ((a >> 16) & 1u)) >> 16;
                hi = (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
            } else {
                lo = __builtin_bit_cast(uint16_t, (_Float16)o[2 * i]);
                hi = __builtin_bit_cast(uint16_t, (_Float16)o[2 * i + 1]);
            }
            w[i] = lo | (hi << 16);
        }
        __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(static_cast<uint16_t*>(Y) + idx));
    }
}

// fp32 results of one step of a wave.  The 64 lanes hold 64 chunks of 8 values (32 bytes each) that are consecutive
// in the output - 2 KB - with chunk `pos` in a lane order of their own; a lane storing its own two 16-byte halves
// makes two instructions that each write every other 16 bytes.  Here the chunks go to LDS in place and are read back in
// lane order: each lane then holds bytes [16 lane, 16 lane + 16) of the first and of the second KB, and each of
// the two store instructions writes 1 KB of consecutive bytes (measured on 4096-wide rows from 4-bit codes: 0.52 of
// the HBM peak with per-lane halves, 0.59 with a quad exchange, 0.8 this way).  `lds`: 2 KB owned by this wave; the
// LDS pipe keeps a wave's instructions in order, so the buffer is reused step after step.  put(e, unit) stores the
// 16-byte unit of values e .. e + 3 of the block where it belongs (and decides whether it exists).  Every lane of the
// wave must be active.
template <typename Put>
__device__ __forceinline__ void store_block_f32(float* lds, int pos, int lane, const float (&v)[8], float k, float add0,
                                                Put put) {
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = v[i] * k;
    o[0] += add0;
    u32x4* const w = reinterpret_cast<u32x4*>(lds) + 2 * pos;
    w[0] = u32x4{__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3])};
    w[1] = u32x4{__float_as_uint(o[4]), __float_as_uint(o[5]), __float_as_uint(o[6]), __float_as_uint(o[7])};
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const u32x4 lo = reinterpret_cast<const u32x4*>(lds)[lane];
    const u32x4 hi = reinterpret_cast<const u32x4*>(lds)[64 + lane];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    put(4 * lane, lo);
    put(256 + 4 * lane, hi);
}

// Squared quantization error of one rotated row for the clip ratios [k0, k1) (sections 2.1, 3.1):
// t = y / Delta_k, r = clamp(round(t)), e = y - r Delta_k, sum e^2 - five vector-ALU operations per
// value and candidate, four candidates at a time (independent chains, interleaved reductions).
// v: the lane's NVAL values of the un-normalised rotated row, carrying the lane's sign `flip`;
// m: the row's absmax.  The sum runs over the lanes that share the row: ROW_BITS lane bits inside a
// DPP row plus the four DPP rows.  emit(k, sum) is called by every lane with the reduced sum.
template <int NVAL, int BITS, int ROW_BITS, typename Emit>
__device__ __forceinline__ void qe_candidates(const float (&v)[NVAL], float m, float flip, const ClipList& clips,
                                              int k0, int k1, Emit emit) {
    constexpr float kQmax = (float)((1 << (BITS - 1)) - 1), kQmin = -(float)(1 << (BITS - 1));
    const double inv_m = m > 0.0f ? 1.0 / (double)m : 0.0;
    for (int kb = k0; kb < k1; kb += 4) {
        float sk[4], ndk[4], e2[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = kb + j < k1 ? kb + j : k1 - 1;
            // 1 / Delta_k = (levels / clip_k) / amax and Delta_k = (clip_k / levels) amax: the
            // row-independent factors come with the clip list, so a candidate costs two fp64 products
            sk[j] = flip * (float)(clips.lvl_over_clip[k] * inv_m);          // lane sign folded in
            ndk[j] = -flip * (float)(clips.clip_over_lvl[k] * (double)m);
            e2[j] = 0.0f;
        }
#pragma unroll
        for (int i = 0; i < NVAL; ++i) {
            const float y = v[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float r = __builtin_amdgcn_fmed3f(__builtin_rintf(y * sk[j]), kQmin, kQmax);
                const float e = fmaf(r, ndk[j], y);
                e2[j] = fmaf(e, e, e2[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) e2[j] += dpp_f<kDppXor1>(e2[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) e2[j] += dpp_f<kDppXor2>(e2[j]);
        if (ROW_BITS >= 3) {
#pragma unroll
            for (int j = 0; j < 4; ++j) e2[j] += dpp_f<kDppHalfMirror>(e2[j]);
        }
        if (ROW_BITS >= 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) e2[j] += dpp_f<kDppRor8>(e2[j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) e2[j] = rows_sum(e2[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kb + j < k1) emit(kb + j, e2[j]);
    }
}

}  // namespace
}  // namespace rq
