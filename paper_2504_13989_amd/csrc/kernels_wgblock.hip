// Workgroup block kernel: bf16 rows of order n = pb * 128 with a +-1 block of order
// 32 < pb <= 256 along the strided axis (H_n = B (x) H_128, B = H_p (x) H_{2^(k-7)}; sections
// 2.3.2, 2.3.3) - e.g. 18944 = 148 * 128 with the order-148 Paley II block.
//
// The dense block product Y1[pb x 128] = B * X[pb x 128] is a real contraction (pb adds per
// output), so it runs on the matrix cores; W = ceil(pb / 32) waves share a row:
//   phase 1  wave w loads block rows 32w .. 32w+31 (16-byte chunks), transposes 16-bit values
//            inside each lane (v_perm_b32) so that 8 consecutive block rows of one column sit in
//            one 16-byte operand, and writes the operands to LDS laid out [column][block row],
//            16-byte units xor-swizzled by the lane's column group so that writes and reads
//            are free of bank conflicts;
//   phase 2  wave w computes output block rows 32w .. 32w+31 for all 128 columns:
//            2 (row halves) x 8 (column tiles) x W (contraction steps) v_mfma_f32_16x16x32_bf16,
//            its 2 W operand tiles of B resident in registers, the data operands read from LDS;
//   phase 3  128-point transform along the columns: three register stages, four fused DPP
//            stages, absmax; workgroup absmax through LDS;
//   phase 4  scale, round/clamp, pack, store (as in the one-wave block kernel).
// Column tile nt holds columns {8 c + nt}, so a lane ends up with 8 consecutive columns of 8
// block rows.  A workgroup loops over rows; two barriers per row order the LDS reuse.
#include "wave_common.h"

namespace rq {
namespace {

template <int W>
constexpr int wg_chunks() { return ((4 * W + 7) / 8) * 8; }   // 16-byte units per LDS column

template <int W, int BITS>
__global__ __launch_bounds__(64 * W) void k_wg_block(WaveArgs a, int pb) {
    constexpr int NCH = wg_chunks<W>();
    extern __shared__ u32x4 lds[];                     // [128 columns][NCH]
    __shared__ float wmax[8];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;    // logical column group (8 columns)
    const int swz = c & 7;

    u32x4 A[2][W];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int kk = 0; kk < W; ++kk) A[h][kk] = a.tiles[((wave * 2 + h) * W + kk) * 64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;

    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const uint16_t* xr = a.X + row * a.ld;
        // ---- phase 1
        u32x4 R[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int ar = 32 * wave + 8 * g + t;
            R[t] = load_chunk(xr, ar * 128 + c * 8, ar < pb ? a.d : 0);
        }
#pragma unroll
        for (int ic = 0; ic < 8; ++ic) {
            u32x4 bm;
            const uint32_t sel = (ic & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                bm[w] = __builtin_amdgcn_perm(R[2 * w + 1][ic >> 1], R[2 * w][ic >> 1], sel);
            lds[(8 * c + ic) * NCH + ((4 * wave + g) ^ swz)] = bm;
        }
        __syncthreads();
        // ---- phase 2
        f32x4 acc[8][2];
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            acc[nt][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc[nt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < W; ++kk) {
                const bf16x8 b8 = __builtin_bit_cast(bf16x8, lds[(8 * c + nt) * NCH + ((4 * kk + g) ^ swz)]);
                acc[nt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[0][kk]), b8, acc[nt][0], 0, 0, 0);
                acc[nt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[1][kk]), b8, acc[nt][1], 0, 0, 0);
            }
        }
        // ---- phase 3
#pragma unroll
        for (int s = 1; s < 8; s <<= 1)
#pragma unroll
            for (int nt = 0; nt < 8; ++nt)
                if (!(nt & s))
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const f32x4 u = acc[nt][h], v = acc[nt | s][h];
                        acc[nt][h] = u + v;
                        acc[nt | s][h] = u - v;
                    }
        float m = 0.0f;
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 v = acc[nt][h];
                lane_stages_fused(v, sf[0], sf[1], sf[2], sf[3]);
                acc[nt][h] = v;
                m = absmax4(m, v);
            }
        m = wave_absmax(m);
        if (lane == 0) wmax[wave] = m;
        __syncthreads();    // also: every wave is done reading this row's operands from LDS
        m = wmax[0];
#pragma unroll
        for (int w = 1; w < W; ++w) m = fmaxf(m, wmax[w]);
        // ---- phase 4
        const float s = m > 0.0f ? flip * (float)(a.c1 / (double)m) : 0.0f;
        uint32_t* out = a.codes + row * (int64_t)(128 * BITS / 32) * pb;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int ip = 0; ip < 4; ++ip) {
                const int ao = 32 * wave + 16 * h + 4 * ip + g;   // output block row of this register
                const uint32_t w = Quant<BITS>::pack8(acc[0][h][ip], acc[1][h][ip], acc[2][h][ip],
                                                      acc[3][h][ip], acc[4][h][ip], acc[5][h][ip],
                                                      acc[6][h][ip], acc[7][h][ip], s);
                const int word = ao * 16 + c;
                if (BITS == 4) {
                    if (ao < pb) store_codes(out + word, w);
                } else {
                    const int qpos = c & 3;
                    const uint32_t dw = merge24<true>(w, qpos);
                    if (ao < pb && qpos < 3) store_codes(out + (word >> 2) * 3 + qpos, dw);
                }
            }
        if (threadIdx.x == 0) a.scales[row] = (float)(a.c2 * (double)m);
    }
}

template <int W>
size_t wg_lds_bytes() { return (size_t)128 * wg_chunks<W>() * 16; }

template <int W>
int launch_w(const rq_hadamard* h, const WaveArgs& a, int bits, int pb, hipStream_t s) {
    const size_t lds = wg_lds_bytes<W>();
    const int per_cu = (int)((size_t)h->max_lds / (lds + 64));
    const int64_t cap = (int64_t)h->num_cu * (per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu));
    const unsigned grid = (unsigned)(a.rows < cap ? a.rows : cap);
    if (bits == 4)
        hipLaunchKernelGGL((k_wg_block<W, 4>), dim3(grid), dim3(64 * W), lds, s, a, pb);
    else
        hipLaunchKernelGGL((k_wg_block<W, 3>), dim3(grid), dim3(64 * W), lds, s, a, pb);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int W>
bool prepare_w() {
    const int lds = (int)wg_lds_bytes<W>();
    if (lds <= 48 * 1024) return true;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k_wg_block<W, 4>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds) == hipSuccess &&
           hipFuncSetAttribute(reinterpret_cast<const void*>(k_wg_block<W, 3>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds) == hipSuccess;
}

}  // namespace

// Operand tiles of the zero-padded block `bm` (order pb) for W = ceil(pb/32) waves:
// [wave][half][kk][lane] x 16 bytes; operand lane (gA, mm) of (wave, half, kk) holds block row
// 32 wave + 16 half + 4 (mm & 3) + (mm >> 2) at the contraction slots a = 32 kk + 8 gA + i.
std::vector<uint32_t> wg_block_tiles(const std::vector<int8_t>& bm, int pb) {
    const int W = (pb + 31) / 32;
    std::vector<uint32_t> t((size_t)W * 2 * W * 64 * 4, 0u);
    for (int w = 0; w < W; ++w)
        for (int hh = 0; hh < 2; ++hh)
            for (int kk = 0; kk < W; ++kk)
                for (int lane = 0; lane < 64; ++lane) {
                    const int gA = lane >> 4, mm = lane & 15;
                    const int ao = 32 * w + 16 * hh + 4 * (mm & 3) + (mm >> 2);
                    for (int i = 0; i < 8; ++i) {
                        const int ai = 32 * kk + 8 * gA + i;
                        uint32_t v = 0;
                        if (ao < pb && ai < pb) v = bm[(size_t)ao * pb + ai] > 0 ? 0x3F80u : 0xBF80u;
                        t[((((size_t)w * 2 + hh) * W + kk) * 64 + lane) * 4 + (i >> 1)] |= v << ((i & 1) * 16);
                    }
                }
    return t;
}

bool wg_block_prepare(int pb) {
    switch ((pb + 31) / 32) {
        case 2: return prepare_w<2>();
        case 3: return prepare_w<3>();
        case 4: return prepare_w<4>();
        case 5: return prepare_w<5>();
        case 6: return prepare_w<6>();
        case 7: return prepare_w<7>();
        case 8: return prepare_w<8>();
        default: return false;
    }
}

bool wg_block_supports(const rq_hadamard* h, const RowArgs& a) {
    if (h->device < 0 || !h->d_tiles || !h->wg_ok || a.dtype != RQ_BF16 || a.p == 1) return false;
    const int pb = a.log2m >= 7 ? (a.p << (a.log2m - 7)) : 0;
    if (pb <= 32 || pb > 256) return false;
    if ((reinterpret_cast<uintptr_t>(a.X) & 15) != 0 || (a.ld & 7) != 0 || (a.d & 7) != 0) return false;
    return true;
}

int wg_block_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                             float* scales, hipStream_t s) {
    const double lvl = (double)((1 << a.bits) - 1);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(h->d_tiles), codes, scales,
               lvl / (double)clip, (double)clip / (std::sqrt((double)a.n) * lvl)};
    const int pb = a.p << (a.log2m - 7);
    switch ((pb + 31) / 32) {
        case 2: return launch_w<2>(h, w, a.bits, pb, s);
        case 3: return launch_w<3>(h, w, a.bits, pb, s);
        case 4: return launch_w<4>(h, w, a.bits, pb, s);
        case 5: return launch_w<5>(h, w, a.bits, pb, s);
        case 6: return launch_w<6>(h, w, a.bits, pb, s);
        case 7: return launch_w<7>(h, w, a.bits, pb, s);
        case 8: return launch_w<8>(h, w, a.bits, pb, s);
        default: return RQ_ERR_NO_ORDER;
    }
}

}  // namespace rq
