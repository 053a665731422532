// Dense-block kernel: bf16 rows of an order n <= 4096 whose factorisation leaves no long
// power-of-two axis for the wave kernels - above all a large Paley block taken over the whole
// dimension (1544 = 1543 + 1, the 1536 + 8 expansion of section 5.2.2), also p * 2^k with k < 7.
// Here the rotation really is a dense contraction, y = H_n x with n multiply-adds per output
// (sections 2.3.3, 4.2), so it runs on the matrix cores as a GEMM: D[a'][row] = sum_a H[a'][a]
// X[row][a], v_mfma_f32_16x16x32_bf16 with
//   B operand  16 rows x 32 inputs straight from memory: lane (g, r) loads the 16 bytes
//              X[row0 + r][32 kk + 8 g ..] (exact bf16, no conversion, no transposition);
//   A operand  a 16 x 32 tile of +-1 (bf16) from a table built with the handle, [kk][mt][lane]: the tiles
//              of one contraction step are contiguous, and all workgroups walk the table in step;
//   D          lane (g, r) register j = output 16 mt + 4 g + j of row r, fp32.
// A workgroup of 8 waves owns 16 rows (32 when there are rows enough: every tile of the table then
// serves two groups of rows); wave w owns the output tiles mt = w, w + 8, ... and keeps
// their accumulators in registers over the whole contraction.  Then: row absmax (registers, the
// four lane rows, the eight waves through LDS), scale, round/clamp (section 2.1 with the clip
// ratio of section 3.1), pack into an LDS image of the 16 packed rows, copy out coalesced.
// The table is read once per workgroup (n^2 / 8 bytes per row): the kernel is bound by that L2
// traffic and the matrix cores, not by HBM.
#include "wave_common.h"

namespace rq {
namespace {

constexpr int kDenseWaves = 8;

template <int MTW, int NT, int BITS>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense_block(WaveArgs a, int n) {
    constexpr int RB = 16 * NT;                          // rows per workgroup
    extern __shared__ __attribute__((aligned(16))) uint8_t stage[];      // RB packed rows
    __shared__ float wmax[kDenseWaves][RB];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, r = lane & 15;
    const int MT = (n + 15) >> 4, KK = (n + 31) >> 5;
    const int row_bytes = n * BITS / 8;
    const int64_t row0 = (int64_t)blockIdx.x * RB;
    bool row_ok[NT];
    const uint16_t* xr[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        const int64_t row = row0 + 16 * q + r;
        row_ok[q] = row < a.rows;
        xr[q] = a.X + (row_ok[q] ? row : 0) * a.ld;
    }

    f32x4 acc[MTW][NT];
#pragma unroll
    for (int j = 0; j < MTW; ++j)
#pragma unroll
        for (int q = 0; q < NT; ++q) acc[j][q] = f32x4{0.f, 0.f, 0.f, 0.f};

    // The contraction is software-pipelined two steps deep: the operands of step kk + 1 are requested
    // before the matrix-core instructions of step kk are issued (two register stages, loop unrolled
    // by two), because a wave otherwise sits out a full memory latency per step with only two waves
    // per SIMD to cover it.  With NT = 2 every operand tile of the table serves two groups of 16 rows.
    u32x4 tA[MTW], tB[MTW], xA[NT], xB[NT];
    auto fetch = [&](int kk, u32x4 (&t)[MTW], u32x4 (&x)[NT]) {
        const int e0 = 32 * kk + 8 * g;
#pragma unroll
        for (int q = 0; q < NT; ++q) {
            const bool in = row_ok[q] && e0 < a.d;       // zero padding beyond d (section 4.2)
            x[q] = load16(xr[q] + (in ? e0 : 0));
            if (!in) x[q] = u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int mt = wave + kDenseWaves * j;
            if (mt < MT) t[j] = a.tiles[((size_t)kk * MT + mt) * 64 + lane];
        }
    };
    auto contract = [&](const u32x4 (&t)[MTW], const u32x4 (&x)[NT]) {
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int mt = wave + kDenseWaves * j;
            if (mt < MT) {
#pragma unroll
                for (int q = 0; q < NT; ++q)
                    acc[j][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t[j]),
                                                                        __builtin_bit_cast(bf16x8, x[q]), acc[j][q], 0, 0, 0);
            }
        }
    };
    fetch(0, tA, xA);
    for (int kk = 0; kk < KK; kk += 2) {
        if (kk + 1 < KK) fetch(kk + 1, tB, xB);
        contract(tA, xA);
        if (kk + 2 < KK) fetch(kk + 2, tA, xA);
        if (kk + 1 < KK) contract(tB, xB);
    }

    // absmax of the lane's rows: this lane's registers, the four lane rows, the eight waves
    float m[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        float v = 0.0f;
#pragma unroll
        for (int j = 0; j < MTW; ++j) v = absmax4(v, acc[j][q]);
        v = __uint_as_float(rows_max_u32(__float_as_uint(v)));
        if (g == 0) wmax[wave][16 * q + r] = v;
    }
    __syncthreads();
    float s[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        float v = wmax[0][16 * q + r];
#pragma unroll
        for (int w = 1; w < kDenseWaves; ++w) v = __builtin_fmaxf(v, wmax[w][16 * q + r]);
        m[q] = v;
        s[q] = v > 0.0f ? (float)(a.c1 / (double)v) : 0.0f;
    }

    // codes of outputs 16 mt + 4 g .. + 3 of a row: 16 bits (b = 4) or 12 bits (b = 3); with 3 bits two
    // neighbouring lane rows make 3 whole bytes
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        const int mt = wave + kDenseWaves * j;
        if (mt < MT) {                                   // wave-uniform
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                uint8_t* srow = stage + (16 * q + r) * row_bytes;
                uint32_t w = 0;
#pragma unroll
                for (int e = 3; e >= 0; --e) {
                    float u = fmaf(acc[j][q][e], s[q], Quant<BITS>::kBias);
                    u = __builtin_amdgcn_fmed3f(u, Quant<BITS>::kLo, Quant<BITS>::kHi);
                    w = (w << BITS) | ((__float_as_uint(u) ^ (1u << (BITS - 1))) & ((1u << BITS) - 1u));
                }
                const int o = 16 * mt + 4 * g;           // first output of this lane
                if (BITS == 4) {
                    if (o < n) *reinterpret_cast<uint16_t*>(srow + o / 2) = (uint16_t)w;
                } else {
                    const uint32_t hi = (uint32_t)__shfl_down((int)w, 16, 64);      // lane row g + 1
                    const uint32_t v = w | (hi << 12);
                    if (!(g & 1) && o < n) {             // n is a multiple of 8: outputs o .. o + 7 exist together
                        uint8_t* p = srow + o * 3 / 8;
                        p[0] = (uint8_t)v;
                        p[1] = (uint8_t)(v >> 8);
                        p[2] = (uint8_t)(v >> 16);
                    }
                }
            }
        }
    }
    __syncthreads();
    // the packed rows of the workgroup are contiguous in the output
    const int64_t left = a.rows - row0;
    const int valid = left < RB ? (int)left : RB;
    const int total = valid * row_bytes;
    uint8_t* out = reinterpret_cast<uint8_t*>(a.codes) + row0 * row_bytes;      // 16 row_bytes | 4-byte aligned
    for (int i = threadIdx.x; i < total / 4; i += blockDim.x)
        reinterpret_cast<uint32_t*>(out)[i] = reinterpret_cast<const uint32_t*>(stage)[i];
    for (int i = (total & ~3) + threadIdx.x; i < total; i += blockDim.x) out[i] = stage[i];
    if (wave == 0 && g == 0) {
#pragma unroll
        for (int q = 0; q < NT; ++q)
            if (row_ok[q]) a.scales[row0 + 16 * q + r] = (float)(a.c2 * (double)m[q]);
    }
}

template <int MTW, int NT>
int launch_dense(const WaveArgs& a, int n, int bits, hipStream_t s) {
    const int64_t groups = (a.rows + 16 * NT - 1) / (16 * NT);
    if (groups > 0x7fffffffLL) return RQ_ERR_ARG;
    const size_t lds = (size_t)16 * NT * n * bits / 8;
    if (bits == 4)
        hipLaunchKernelGGL((k_dense_block<MTW, NT, 4>), dim3((unsigned)groups), dim3(64 * kDenseWaves), lds, s, a, n);
    else
        hipLaunchKernelGGL((k_dense_block<MTW, NT, 3>), dim3((unsigned)groups), dim3(64 * kDenseWaves), lds, s, a, n);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace

// Matrix-core operand table of the whole n x n matrix `hm` (row-major +-1): [kk][mt][lane] x 16
// bytes; operand lane (gA, mm) of tile (mt, kk) holds H[16 mt + mm][32 kk + 8 gA + i], i = 0..7, as
// bf16, zero outside the matrix.
std::vector<uint32_t> dense_block_tiles(const std::vector<int8_t>& hm, int n) {
    const int MT = (n + 15) / 16, KK = (n + 31) / 32;
    std::vector<uint32_t> t((size_t)MT * KK * 64 * 4, 0u);
    for (int mt = 0; mt < MT; ++mt)
        for (int kk = 0; kk < KK; ++kk)
            for (int lane = 0; lane < 64; ++lane) {
                const int gA = lane >> 4, mm = lane & 15;
                const int ao = 16 * mt + mm;
                for (int i = 0; i < 8; ++i) {
                    const int ai = 32 * kk + 8 * gA + i;
                    uint32_t v = 0;
                    if (ao < n && ai < n) v = hm[(size_t)ao * n + ai] > 0 ? 0x3F80u : 0xBF80u;
                    t[(((size_t)kk * MT + mt) * 64 + lane) * 4 + (i >> 1)] |= v << ((i & 1) * 16);
                }
            }
    return t;
}

bool dense_block_supports(const rq_hadamard* h, const RowArgs& a) {
    if (h->device < 0 || !h->d_tiles || !h->dense_ok || a.dtype != RQ_BF16) return false;
    if ((reinterpret_cast<uintptr_t>(a.X) & 15) != 0 || (a.ld & 7) != 0 || (a.d & 7) != 0) return false;
    return true;
}

int dense_block_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                                float* scales, hipStream_t s) {
    const double lvl = (double)((1 << a.bits) - 1);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(h->d_tiles), codes, scales,
               lvl / (double)clip, (double)clip / (std::sqrt((double)a.n) * lvl)};
    const int mtw = ((a.n + 15) / 16 + kDenseWaves - 1) / kDenseWaves;
    // 32 rows per workgroup halve the traffic of the operand table; used when that still leaves a
    // workgroup for every CU and the accumulators fit the register budget (two waves per SIMD)
    const bool two = a.rows >= (int64_t)32 * h->num_cu && mtw <= 13;
    if (mtw <= 4) return two ? launch_dense<4, 2>(w, a.n, a.bits, s) : launch_dense<4, 1>(w, a.n, a.bits, s);
    if (mtw <= 8) return two ? launch_dense<8, 2>(w, a.n, a.bits, s) : launch_dense<8, 1>(w, a.n, a.bits, s);
    if (mtw <= 13) return two ? launch_dense<13, 2>(w, a.n, a.bits, s) : launch_dense<13, 1>(w, a.n, a.bits, s);
    if (mtw <= 16) return launch_dense<16, 1>(w, a.n, a.bits, s);
    if (mtw <= 32) return launch_dense<32, 1>(w, a.n, a.bits, s);
    return RQ_ERR_NO_ORDER;
}

}  // namespace rq
