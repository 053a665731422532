// Rotation alone on the wave path: Y = (H_n pad(x) / sqrt(n))[:d_out] for 16-bit rows of Sylvester
// order n = 128 ... 8192 (sections 2.2, 2.3.2), written as bf16, fp16 or fp32.  This is the online
// rotation of a tensor that is not quantized afterwards - the query heads, which must carry the same
// per-head H_128 as the keys whose rotated form goes into the quantized cache - so it gets the same
// treatment as rotate_quantize: one wave per row (n >= 1024) or 16 >> CB rows per wave pass
// (n = 32 << CB), five stages on the matrix cores, the rest in registers and DPP, 16-byte loads and
// stores (fp32 results pass through LDS first, so that every store instruction covers 1 KB of consecutive
// bytes: store_block_f32).  H_{2^k} is symmetric, so the transposed product is the same kernel.
//
// The same kernels take packed codes instead of rows (rq_dequantize_rotate: x = H^T (code Delta) / sqrt(n),
// sections 2.1, 2.3): a b-bit code u (offset binary) becomes the bf16 pattern 0x4300 | u = 128 + u by bit
// operations alone, so the matrix cores transform K + q with K = 128 + 2^(b-1) (K = 128 for the unsigned
// group codes) exactly in integers; H (K 1) = n K e_0, so the constant comes back out of output element 0
// of the row, and Delta / sqrt(n) multiplies once at the end.  For the asymmetric group codes with one
// group per row (n = 128, the KV head rows) the group offset lo adds lo sqrt(n) to element 0.
#include "wave_common.h"

namespace rq {
namespace {

struct RotArgs {
    const uint16_t* X;
    int64_t rows;
    int d;
    int64_t ld;
    const u32x4* tiles;
    void* Y;
    int d_out;
    int64_t ld_out;
    float inv;            // 1 / sqrt(n)
    // packed codes as the source (SRC = 3, 4: bits per code), else null
    const uint32_t* codes = nullptr;
    const float* scales = nullptr;
    const float* mins = nullptr;      // asymmetric group codes, one group per row (n = 128)
    float sqrt_n = 0.0f;
};

// The lane's 8 consecutive codes (group idx of the row: codes 8 idx .. 8 idx + 7) as a matrix-core
// operand: four dwords of two bf16 patterns 0x4300 | u each.  Signed codes are two's complement fields:
// one xor makes them offset binary.  A 3-bit group is 24 bits at byte 3 idx: the dword it starts in and,
// where it continues there, the next one (lanes whose field ends inside the first dword read that one
// twice, so nothing beyond the row is touched).  CodeLane holds what depends on the lane alone.
struct CodeLane {
    uint32_t off0, off1;      // byte offsets of the two dwords from the group-0 position
    uint32_t sh;              // bit position of the field in the first dword
};
template <int BITS>
__device__ __forceinline__ CodeLane code_lane(int idx) {
    if constexpr (BITS == 4) return CodeLane{(uint32_t)idx * 4u, 0u, 0u};
    const uint32_t byte = 3u * (uint32_t)idx, sh = (byte & 3u) * 8u;
    const uint32_t off0 = byte & ~3u;
    return CodeLane{off0, off0 + (sh >= 16u ? 4u : 0u), sh};
}
// base: the packed codes at the lane-independent part of the position (uniform where the wave works on one row)
template <int BITS, bool ASYM>
__device__ __forceinline__ u32x4 code_operand(const uint32_t* base, const CodeLane& cl) {
    const char* p = reinterpret_cast<const char*>(base);
    uint32_t w;
    if constexpr (BITS == 4) {
        w = *reinterpret_cast<const uint32_t*>(p + cl.off0);
        if (!ASYM) w ^= 0x88888888u;
    } else {
        const uint32_t lo = *reinterpret_cast<const uint32_t*>(p + cl.off0);
        const uint32_t hi = *reinterpret_cast<const uint32_t*>(p + cl.off1);
        w = __builtin_amdgcn_alignbit(hi, lo, cl.sh);
        if (!ASYM) w ^= 0x924924u;
    }
    u32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if constexpr (BITS == 4) {
            const uint32_t by = (w >> (8 * j)) & 0xffu;                 // two codes
            r[j] = ((by * 0x1001u) & 0x000f000fu) | 0x43004300u;
        } else {
            const uint32_t six = (w >> (6 * j)) & 0x3fu;
            r[j] = ((six * 0x2001u) & 0x00070007u) | 0x43004300u;
        }
    }
    return r;
}

// n = 512 T: one wave per row.
template <int T, bool F16, int OUT, int SRC = 0>
__global__ __launch_bounds__(64) void k_wave_rotate(RotArgs a) {
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;
    const int chunk = (g << 4) + c;
    __shared__ __attribute__((aligned(16))) float lds_out[OUT == 1 ? 512 : 4];   // fp32 results pass through LDS, see store_block_f32
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    float k = ((__builtin_popcount(c) & 1) ? -1.0f : 1.0f) * a.inv;
    constexpr int ROW_DWORDS = SRC ? 512 * T * SRC / 32 : 0;
    // packed codes: the constant K = 128 + 2^(b-1) of the patterns leaves through element 0 of the row
    const float corr = (SRC && chunk == 0) ? -(float)(512 * T) * (float)(128 + (1 << (SRC ? SRC - 1 : 0))) : 0.0f;
    const float sgn = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;
    const CodeLane cl = code_lane<SRC ? SRC : 4>(chunk);
    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        f32x4 acc[T][2];
        u32x4 raw[T];
        if constexpr (SRC == 0) {
            const RowView xv = row_view(a.X + row * a.ld, a.d);
#pragma unroll
            for (int t = 0; t < T; ++t) raw[t] = load_chunk(xv, (t * 64 + chunk) * 8);
        } else {
            const uint32_t* cr = a.codes + row * (int64_t)ROW_DWORDS;
#pragma unroll
            for (int t = 0; t < T; ++t) raw[t] = code_operand<SRC ? SRC : 4, false>(cr + t * (ROW_DWORDS / T), cl);
            k = sgn * a.inv * a.scales[row];
        }
        __builtin_amdgcn_sched_barrier(0);              // every load is issued before the first wait
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            acc[t][0] = mfma_pm1<F16 && SRC == 0>(A0, raw[t], z);
            acc[t][1] = mfma_pm1<F16 && SRC == 0>(A1, raw[t], z);
        }
#pragma unroll
        for (int s = 1; s < T; s <<= 1)
#pragma unroll
            for (int t = 0; t < T; ++t)
                if (!(t & s))
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const f32x4 u = acc[t][h], v = acc[t | s][h];
                        acc[t][h] = u + v;
                        acc[t | s][h] = u - v;
                    }
#pragma unroll
        for (int t = 0; t < T; ++t) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 v = acc[t][h];
                lane_stages_fused(v, sf[0], sf[1], sf[2], sf[3]);
                acc[t][h] = v;
            }
            if (SRC && t == 0) acc[0][0][0] += corr;
            const int col = (t * 64 + chunk) * 8;
            const float v8[8] = {acc[t][0][0], acc[t][0][1], acc[t][0][2], acc[t][0][3],
                                 acc[t][1][0], acc[t][1][1], acc[t][1][2], acc[t][1][3]};
            if constexpr (OUT == 1) {
                float* const yr = static_cast<float*>(a.Y) + row * a.ld_out + t * 512;
                store_block_f32(lds_out, chunk, lane, v8, k, 0.0f, [&](int e, const u32x4& unit) {
                    if (t * 512 + e < a.d_out) __builtin_nontemporal_store(unit, reinterpret_cast<u32x4*>(yr + e));
                });
            } else if (col < a.d_out) {
                store8<OUT>(a.Y, row * a.ld_out + col, v8, k);
            }
        }
    }
}

// n = 32 << CB (128, 256, 512): 16 >> CB rows per wave pass, U passes in flight.
template <int CB, int U, bool F16, int OUT, int SRC = 0, bool ASYM = false>
__global__ __launch_bounds__(64) void k_wave_rotate_short(RotArgs a) {
    static_assert(!ASYM || (SRC != 0 && CB == 2), "group codes: one group per row");
    constexpr int RPW = 16 >> CB;
    constexpr int ROW_DWORDS = SRC ? (32 << CB) * SRC / 32 : 0;
    constexpr int SUPER = RPW * U;
    const int lane = threadIdx.x;
    const int g = lane >> 4, nnl = lane & 15;
    const int cphys = nnl & ((1 << CB) - 1);
    const int rsub = nnl >> CB;
    const int c = (CB >= 3 && (cphys & 4)) ? (cphys ^ 3) : cphys;
    const int chunk = (g << CB) + c;
    __shared__ __attribute__((aligned(16))) float lds_out[OUT == 1 ? 512 : 4];   // fp32 results pass through LDS, see store_block_f32
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const uint32_t sg0 = (c & 1) ? 0x80000000u : 0u;
    const float k0 = ((__builtin_popcount(c >> 1) & 1) ? -1.0f : 1.0f) * a.inv;  // stages 2.. are the fused ones
    // packed codes: the constant of the patterns (128, plus 2^(b-1) for signed codes) leaves through element 0
    const float corr = (SRC && chunk == 0) ? -(float)(32 << CB) * (float)(128 + (ASYM ? 0 : 1 << (SRC ? SRC - 1 : 0))) : 0.0f;
    const CodeLane cl = code_lane<SRC ? SRC : 4>(chunk);
    const int64_t n_super = (a.rows + SUPER - 1) / SUPER;
    for (int64_t sgi = blockIdx.x; sgi < n_super; sgi += gridDim.x) {
        const int64_t row0 = sgi * SUPER;
        u32x4 raw[U];
        float ks[U], add0[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = row0 + u * RPW + rsub;
            if constexpr (SRC == 0) {
                const bool in = row < a.rows && chunk * 8 < a.d;
                raw[u] = load16(a.X + (in ? row * a.ld + chunk * 8 : 0));
                ks[u] = k0;
                add0[u] = 0.0f;
            } else {
                const int64_t rl = row < a.rows ? row : a.rows - 1;      // rows beyond the end: loads only
                raw[u] = code_operand<SRC ? SRC : 4, ASYM>(a.codes + rl * ROW_DWORDS, cl);
                ks[u] = k0 * a.scales[rl];
                add0[u] = (ASYM && chunk == 0) ? a.mins[rl] * a.sqrt_n : 0.0f;
            }
        }
        __builtin_amdgcn_sched_barrier(0);              // every load is issued before the first wait
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = row0 + u * RPW + rsub;
            if (SRC == 0 && !(row < a.rows && chunk * 8 < a.d)) raw[u] = u32x4{0u, 0u, 0u, 0u};
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            f32x4 v0 = mfma_pm1<F16 && SRC == 0>(A0, raw[u], z);
            f32x4 v1 = mfma_pm1<F16 && SRC == 0>(A1, raw[u], z);
            lane_stage<kDppXor1>(v0, sg0);              // compiler-visible first consumer of the matrix-core result
            lane_stage<kDppXor1>(v1, sg0);
            lane_stages_tail<CB>(v0, sf);
            lane_stages_tail<CB>(v1, sf);
            const float v8[8] = {v0[0] + corr, v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
            if constexpr (OUT == 1) {
                // the pass's RPW rows are one block of 64 chunks: row rsub, chunk `chunk`
                const int64_t prow0 = row0 + u * RPW;
                store_block_f32(lds_out, rsub * (4 << CB) + chunk, lane, v8, ks[u], add0[u], [&](int e, const u32x4& unit) {
                    const int64_t orow = prow0 + (e >> (5 + CB));
                    const int ocol = e & ((32 << CB) - 1);
                    if (orow < a.rows && ocol < a.d_out)
                        __builtin_nontemporal_store(unit, reinterpret_cast<u32x4*>(static_cast<float*>(a.Y) + orow * a.ld_out + ocol));
                });
            } else if (row < a.rows && chunk * 8 < a.d_out) {
                store8<OUT>(a.Y, row * a.ld_out + chunk * 8, v8, ks[u], add0[u]);
            }
        }
    }
}

template <int T>
void launch_long(const RotArgs& a, bool f16, int out, unsigned grid, hipStream_t s) {
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, a); };
    if (f16) {
        if (out == 0) go(k_wave_rotate<T, true, 0>); else if (out == 1) go(k_wave_rotate<T, true, 1>); else go(k_wave_rotate<T, true, 2>);
    } else {
        if (out == 0) go(k_wave_rotate<T, false, 0>); else if (out == 1) go(k_wave_rotate<T, false, 1>); else go(k_wave_rotate<T, false, 2>);
    }
}

template <int CB>
void launch_short(const RotArgs& a, bool f16, int out, hipStream_t s) {
    constexpr int U = 4;
    const int64_t items = (a.rows + (16 >> CB) * U - 1) / ((16 >> CB) * U);
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(items < cap ? items : cap);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, a); };
    if (f16) {
        if (out == 0) go(k_wave_rotate_short<CB, U, true, 0>); else if (out == 1) go(k_wave_rotate_short<CB, U, true, 1>); else go(k_wave_rotate_short<CB, U, true, 2>);
    } else {
        if (out == 0) go(k_wave_rotate_short<CB, U, false, 0>); else if (out == 1) go(k_wave_rotate_short<CB, U, false, 1>); else go(k_wave_rotate_short<CB, U, false, 2>);
    }
}

template <int T>
void launch_long_codes(const RotArgs& a, int bits, int out, unsigned grid, hipStream_t s) {
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, a); };
    if (bits == 4) {
        if (out == 0) go(k_wave_rotate<T, false, 0, 4>); else if (out == 1) go(k_wave_rotate<T, false, 1, 4>); else go(k_wave_rotate<T, false, 2, 4>);
    } else {
        if (out == 0) go(k_wave_rotate<T, false, 0, 3>); else if (out == 1) go(k_wave_rotate<T, false, 1, 3>); else go(k_wave_rotate<T, false, 2, 3>);
    }
}

template <int CB, bool ASYM>
void launch_short_codes(const RotArgs& a, int bits, int out, hipStream_t s) {
    constexpr int U = 4;
    const int64_t items = (a.rows + (16 >> CB) * U - 1) / ((16 >> CB) * U);
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(items < cap ? items : cap);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, a); };
    if (bits == 4) {
        if (out == 0) go(k_wave_rotate_short<CB, U, false, 0, 4, ASYM>); else if (out == 1) go(k_wave_rotate_short<CB, U, false, 1, 4, ASYM>); else go(k_wave_rotate_short<CB, U, false, 2, 4, ASYM>);
    } else {
        if (out == 0) go(k_wave_rotate_short<CB, U, false, 0, 3, ASYM>); else if (out == 1) go(k_wave_rotate_short<CB, U, false, 1, 3, ASYM>); else go(k_wave_rotate_short<CB, U, false, 2, 3, ASYM>);
    }
}

}  // namespace

// Packed codes back to rows on the wave path: Sylvester orders 128 .. 8192 (H symmetric: one kernel for
// H and H^T), signed per-token codes, or unsigned group codes when a row is one group (n = 128).
bool wave_dequant_rotate_supports(const rq_hadamard* h, const RowArgs& a, const float* mins, const OutArgs& o) {
    if (h->device < 0 || !h->d_tiles || a.p != 1 || a.log2m < 7 || a.log2m > 13) return false;
    if (mins && a.log2m != 7) return false;
    if ((reinterpret_cast<uintptr_t>(o.Y) & 15) != 0 || (o.d_out & 7) != 0) return false;
    return o.dtype == RQ_F32 ? (o.ld_out & 3) == 0 : (o.ld_out & 7) == 0;
}

int wave_dequant_rotate(const rq_hadamard* h, const RowArgs& a, const uint32_t* codes, const float* scales,
                        const float* mins, const OutArgs& o, hipStream_t s) {
    RotArgs r{nullptr, a.rows, a.n, a.n, static_cast<const u32x4*>(h->d_tiles), o.Y, o.d_out, o.ld_out,
              (float)(1.0 / std::sqrt((double)a.n))};
    r.codes = codes;
    r.scales = scales;
    r.mins = mins;
    r.sqrt_n = (float)std::sqrt((double)a.n);
    const int out = o.dtype == RQ_BF16 ? 0 : o.dtype == RQ_F32 ? 1 : 2;
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(a.rows < cap ? a.rows : cap);
    switch (a.log2m) {
        case 7:
            if (mins) launch_short_codes<2, true>(r, a.bits, out, s);
            else launch_short_codes<2, false>(r, a.bits, out, s);
            break;
        case 8: launch_short_codes<3, false>(r, a.bits, out, s); break;
        case 9: launch_short_codes<4, false>(r, a.bits, out, s); break;
        case 10: launch_long_codes<2>(r, a.bits, out, grid, s); break;
        case 11: launch_long_codes<4>(r, a.bits, out, grid, s); break;
        case 12: launch_long_codes<8>(r, a.bits, out, grid, s); break;
        case 13: launch_long_codes<16>(r, a.bits, out, grid, s); break;
        default: return RQ_ERR_NO_ORDER;
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

bool wave_rotate_supports(const rq_hadamard* h, const RowArgs& a, const OutArgs& o) {
    if (h->device < 0 || !h->d_tiles || a.p != 1 || a.log2m < 7 || a.log2m > 13) return false;
    if (a.dtype != RQ_BF16 && !(a.dtype == RQ_F16 && h->d_tiles_f16)) return false;
    if ((reinterpret_cast<uintptr_t>(a.X) & 15) != 0 || (a.ld & 7) != 0 || (a.d & 7) != 0) return false;
    if ((reinterpret_cast<uintptr_t>(o.Y) & 15) != 0 || (o.d_out & 7) != 0) return false;
    return o.dtype == RQ_F32 ? (o.ld_out & 3) == 0 : (o.ld_out & 7) == 0;
}

int wave_rotate(const rq_hadamard* h, const RowArgs& a, const OutArgs& o, hipStream_t s) {
    const bool f16 = a.dtype == RQ_F16;
    const RotArgs r{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
                    static_cast<const u32x4*>(f16 ? h->d_tiles_f16 : h->d_tiles), o.Y, o.d_out, o.ld_out,
                    (float)(1.0 / std::sqrt((double)a.n))};
    const int out = o.dtype == RQ_BF16 ? 0 : o.dtype == RQ_F32 ? 1 : 2;
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(a.rows < cap ? a.rows : cap);
    switch (a.log2m) {
        case 7: launch_short<2>(r, f16, out, s); break;
        case 8: launch_short<3>(r, f16, out, s); break;
        case 9: launch_short<4>(r, f16, out, s); break;
        case 10: launch_long<2>(r, f16, out, grid, s); break;
        case 11: launch_long<4>(r, f16, out, grid, s); break;
        case 12: launch_long<8>(r, f16, out, grid, s); break;
        case 13: launch_long<16>(r, f16, out, grid, s); break;
        default: return RQ_ERR_NO_ORDER;
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace rq
