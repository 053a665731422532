// One-wave block kernel for blocks of order 32 < pb <= 64: 16-bit rows of order n = pb * 128 <= 8192
// (5120 = 40 * 128, 6144, 7168 ...; H_n = B (x) H_128, B = H_p (x) H_{2^(k-7)}; sections 2.3.2,
// 2.3.3).  The structure is that of the one-wave kernel for pb <= 32 (index layout [ a | c | i ],
// lane (g, c) loads whole 16-byte chunks of several block rows, transposes 16-bit values inside the
// lane into per-column matrix-core operands), with two contraction steps of 32 block rows and up to
// four output tiles of 16 block rows: per column position i, 2 x ceil(pb / 16) matrix-core
// instructions whose accumulators (8 x NV registers, NV = ceil(pb / 4)) then go through the same
// register / DPP butterflies, absmax, quantizer and packer.  The row stays in one wave's registers
// (about 200 of them, two waves per SIMD), so there is no LDS traffic and no barrier as in the
// workgroup kernel that served these orders before.
#include "wave_common.h"

namespace rq {
namespace {

template <int BITS, bool FULL, int NV, bool F16>
__global__ __launch_bounds__(64) void k_wave_block2(WaveArgs a, int pb) {
    static_assert(NV > 8 && NV <= 16, "blocks of 33 .. 64");
    constexpr int MT = (NV + 3) / 4;                      // output tiles of 16 block rows
    __shared__ __attribute__((aligned(16))) uint8_t stage[BITS == 3 ? 64 * 48 : 16];
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;     // logical column chunk
    u32x4 A[MT][2];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) A[m][kk] = a.tiles[(m * 2 + kk) * 64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;

    // contraction step 0: block rows 8 g .. 8 g + 7; step 1: 32 + 8 g .. + 7, moved down to end at
    // pb - 1 where it would run past the block (the operand tiles have zero columns for the
    // duplicates this creates)
    const int base1 = 32 + 8 * g < pb - 8 ? 32 + 8 * g : pb - 8;
    const int e0 = 8 * g * 128 + c * 8, e1 = base1 * 128 + c * 8;
    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const uint16_t* xr = a.X + row * a.ld;
        const RowView xv = row_view(xr, a.d);
        u32x4 R0[8], R1[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) R0[t] = FULL ? load16(xr + e0 + t * 128) : load_chunk(xv, e0 + t * 128);
#pragma unroll
        for (int t = 0; t < 8; ++t) R1[t] = FULL ? load16(xr + e1 + t * 128) : load_chunk(xv, e1 + t * 128);
        __builtin_amdgcn_sched_barrier(0);              // every load is issued before the first wait
        float y[8][NV];
#pragma unroll
        for (int ic = 0; ic < 8; ++ic) {
            u32x4 b0, b1;
            const uint32_t sel = (ic & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                b0[w] = __builtin_amdgcn_perm(R0[2 * w + 1][ic >> 1], R0[2 * w][ic >> 1], sel);
                b1[w] = __builtin_amdgcn_perm(R1[2 * w + 1][ic >> 1], R1[2 * w][ic >> 1], sel);
            }
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                f32x4 d = mfma_pm1<F16>(A[m][0], b0, z);
                d = mfma_pm1<F16>(A[m][1], b1, d);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (4 * m + j < NV) y[ic][4 * m + j] = d[j];
            }
        }
#pragma unroll
        for (int s = 1; s < 8; s <<= 1)
#pragma unroll
            for (int ic = 0; ic < 8; ++ic)
                if (!(ic & s))
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        const float u = y[ic][j], v = y[ic | s][j];
                        y[ic][j] = u + v;
                        y[ic | s][j] = u - v;
                    }
        float mx = 0.0f;
#pragma unroll
        for (int ic = 0; ic < 8; ++ic) {
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (4 * m + 4 <= NV) fused_group<4>(&y[ic][4 * m], sf);
                else if (NV - 4 * m == 3) fused_group<3>(&y[ic][4 * m], sf);
                else if (NV - 4 * m == 2) fused_group<2>(&y[ic][4 * m], sf);
                else fused_group<1>(&y[ic][4 * m], sf);
            }
#pragma unroll
            for (int j = 0; j < NV; ++j) mx = __builtin_fmaxf(mx, __builtin_fabsf(y[ic][j]));
        }
        const float m = wave_absmax<4>(mx);
        const float s = m > 0.0f ? flip * (float)(a.c1 / (double)m) : 0.0f;
        const float scale = (float)(a.c2 * (double)m);

        uint32_t* out = a.codes + row * (int64_t)(128 * BITS / 32) * pb;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int ao = 4 * j + g;                      // output block row of this register
            const uint32_t w = Quant<BITS>::pack8(y[0][j], y[1][j], y[2][j], y[3][j], y[4][j], y[5][j],
                                                  y[6][j], y[7][j], s);
            const int word = ao * 16 + c;
            if (BITS == 4) {
                if (ao < pb) store_codes(out + word, w);
            } else {
                stage24(stage, word, w);                   // block rows >= pb land beyond the copied part
            }
        }
        if (BITS == 3) {
            __syncthreads();
            copy_out16<64 * 3>(stage, out, pb * 3, lane);
            __syncthreads();
        }
        if (lane == 0) a.scales[row] = scale;
    }
}

template <int NV>
void launch_nv(const WaveArgs& w, int bits, bool full, unsigned grid, int pb, hipStream_t s) {
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, w, pb); };
    if (w.f16) {
        if (bits == 4) { if (full) go(k_wave_block2<4, true, NV, true>); else go(k_wave_block2<4, false, NV, true>); }
        else { if (full) go(k_wave_block2<3, true, NV, true>); else go(k_wave_block2<3, false, NV, true>); }
    } else {
        if (bits == 4) { if (full) go(k_wave_block2<4, true, NV, false>); else go(k_wave_block2<4, false, NV, false>); }
        else { if (full) go(k_wave_block2<3, true, NV, false>); else go(k_wave_block2<3, false, NV, false>); }
    }
}

}  // namespace

// Operand tiles of the block `bm` (order 32 < pb <= 64): [tile m][step kk][lane] x 16 bytes.  Operand lane
// (gA, mm) of tile m holds block row 16 m + 4 (mm & 3) + (mm >> 2); its contraction slots i = 0..7 of
// step kk carry input block row 8 gA + i (kk = 0) or min(32 + 8 gA, pb - 8) + i (kk = 1), the latter
// counting only from 32 + 8 gA on (below that it duplicates a row of the previous slot group).
std::vector<uint32_t> wave_block2_tiles(const std::vector<int8_t>& bm, int pb) {
    std::vector<uint32_t> t((size_t)4 * 2 * 64 * 4, 0u);
    for (int m = 0; m < 4; ++m)
        for (int kk = 0; kk < 2; ++kk)
            for (int lane = 0; lane < 64; ++lane) {
                const int gA = lane >> 4, mm = lane & 15;
                const int ao = 16 * m + 4 * (mm & 3) + (mm >> 2);
                const int first = kk == 0 ? 8 * gA : 32 + 8 * gA;
                const int base = kk == 0 ? first : (first < pb - 8 ? first : pb - 8);
                for (int i = 0; i < 8; ++i) {
                    const int ai = base + i;
                    uint32_t v = 0;
                    if (ao < pb && ai >= first && ai < pb) v = bm[(size_t)ao * pb + ai] > 0 ? 0x3F80u : 0xBF80u;
                    t[(((size_t)m * 2 + kk) * 64 + lane) * 4 + (i >> 1)] |= v << ((i & 1) * 16);
                }
            }
    return t;
}

bool wave_block2_supports(const rq_hadamard* h, const RowArgs& a) {
    if (h->device < 0 || !h->d_tiles2 || a.p == 1 || a.log2m < 7) return false;
    if (a.dtype != RQ_BF16 && !(a.dtype == RQ_F16 && h->d_tiles2_f16)) return false;
    const int pb = a.p << (a.log2m - 7);
    if (pb <= 32 || pb > 64) return false;
    if ((reinterpret_cast<uintptr_t>(a.X) & 15) != 0 || (a.ld & 7) != 0 || (a.d & 7) != 0) return false;
    return true;
}

int wave_block2_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                                float* scales, hipStream_t s) {
    const bool f16 = a.dtype == RQ_F16;
    const double lvl = (double)((1 << a.bits) - 1);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(f16 ? h->d_tiles2_f16 : h->d_tiles2), codes, scales,
               lvl / (double)clip, (double)clip / (std::sqrt((double)a.n) * lvl)};
    w.f16 = f16;
    const int pb = a.p << (a.log2m - 7);
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(a.rows < cap ? a.rows : cap);
    const bool full = a.d == a.n;
    switch ((pb + 3) / 4) {
        case 9: launch_nv<9>(w, a.bits, full, grid, pb, s); break;
        case 10: launch_nv<10>(w, a.bits, full, grid, pb, s); break;
        case 11: launch_nv<11>(w, a.bits, full, grid, pb, s); break;
        case 12: launch_nv<12>(w, a.bits, full, grid, pb, s); break;
        case 13: launch_nv<13>(w, a.bits, full, grid, pb, s); break;
        case 14: launch_nv<14>(w, a.bits, full, grid, pb, s); break;
        case 15: launch_nv<15>(w, a.bits, full, grid, pb, s); break;
        case 16: launch_nv<16>(w, a.bits, full, grid, pb, s); break;
        default: return RQ_ERR_NO_ORDER;
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace rq
