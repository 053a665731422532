// Rotation alone on the wave path: Y = (H_n pad(x) / sqrt(n))[:d_out] for 16-bit rows of Sylvester
// order n = 128 ... 8192 (sections 2.2, 2.3.2), written as bf16, fp16 or fp32.  This is the online
// rotation of a tensor that is not quantized afterwards - the query heads, which must carry the same
// per-head H_128 as the keys whose rotated form goes into the quantized cache - so it gets the same
// treatment as rotate_quantize: one wave per row (n >= 1024) or 16 >> CB rows per wave pass
// (n = 32 << CB), five stages on the matrix cores, the rest in registers and DPP, 16-byte loads and
// stores.  H_{2^k} is symmetric, so the transposed product is the same kernel.
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
};

// Eight consecutive results of a lane (carrying the lane's sign in `k`) to columns col .. col + 7.
// OUT: 0 bf16, 1 fp32, 2 fp16 (round to nearest even).
template <int OUT>
__device__ __forceinline__ void store8(void* Y, int64_t idx, const float (&v)[8], float k) {
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = v[i] * k;
    if constexpr (OUT == 1) {
        u32x4* p = reinterpret_cast<u32x4*>(static_cast<float*>(Y) + idx);
        __builtin_nontemporal_store(u32x4{__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3])}, p);
        __builtin_nontemporal_store(u32x4{__float_as_uint(o[4]), __float_as_uint(o[5]), __float_as_uint(o[6]), __float_as_uint(o[7])}, p + 1);
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

// n = 512 T: one wave per row.
template <int T, bool F16, int OUT>
__global__ __launch_bounds__(64) void k_wave_rotate(RotArgs a) {
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;
    const int chunk = (g << 4) + c;
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float k = ((__builtin_popcount(c) & 1) ? -1.0f : 1.0f) * a.inv;
    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const RowView xv = row_view(a.X + row * a.ld, a.d);
        f32x4 acc[T][2];
        u32x4 raw[T];
#pragma unroll
        for (int t = 0; t < T; ++t) raw[t] = load_chunk(xv, (t * 64 + chunk) * 8);
        __builtin_amdgcn_sched_barrier(0);              // every load is issued before the first wait
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            acc[t][0] = mfma_pm1<F16>(A0, raw[t], z);
            acc[t][1] = mfma_pm1<F16>(A1, raw[t], z);
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
            const int col = (t * 64 + chunk) * 8;
            if (col < a.d_out) {
                const float v8[8] = {acc[t][0][0], acc[t][0][1], acc[t][0][2], acc[t][0][3],
                                     acc[t][1][0], acc[t][1][1], acc[t][1][2], acc[t][1][3]};
                store8<OUT>(a.Y, row * a.ld_out + col, v8, k);
            }
        }
    }
}

// n = 32 << CB (128, 256, 512): 16 >> CB rows per wave pass, U passes in flight.
template <int CB, int U, bool F16, int OUT>
__global__ __launch_bounds__(64) void k_wave_rotate_short(RotArgs a) {
    constexpr int RPW = 16 >> CB;
    constexpr int SUPER = RPW * U;
    const int lane = threadIdx.x;
    const int g = lane >> 4, nnl = lane & 15;
    const int cphys = nnl & ((1 << CB) - 1);
    const int rsub = nnl >> CB;
    const int c = (CB >= 3 && (cphys & 4)) ? (cphys ^ 3) : cphys;
    const int chunk = (g << CB) + c;
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const uint32_t sg0 = (c & 1) ? 0x80000000u : 0u;
    const float k = ((__builtin_popcount(c >> 1) & 1) ? -1.0f : 1.0f) * a.inv;   // stages 2.. are the fused ones
    const int64_t n_super = (a.rows + SUPER - 1) / SUPER;
    for (int64_t sgi = blockIdx.x; sgi < n_super; sgi += gridDim.x) {
        const int64_t row0 = sgi * SUPER;
        u32x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = row0 + u * RPW + rsub;
            const bool in = row < a.rows && chunk * 8 < a.d;
            raw[u] = load16(a.X + (in ? row * a.ld + chunk * 8 : 0));
        }
        __builtin_amdgcn_sched_barrier(0);              // every load is issued before the first wait
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = row0 + u * RPW + rsub;
            if (!(row < a.rows && chunk * 8 < a.d)) raw[u] = u32x4{0u, 0u, 0u, 0u};
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            f32x4 v0 = mfma_pm1<F16>(A0, raw[u], z);
            f32x4 v1 = mfma_pm1<F16>(A1, raw[u], z);
            lane_stage<kDppXor1>(v0, sg0);              // compiler-visible first consumer of the matrix-core result
            lane_stage<kDppXor1>(v1, sg0);
            lane_stages_tail<CB>(v0, sf);
            lane_stages_tail<CB>(v1, sf);
            if (row < a.rows && chunk * 8 < a.d_out) {
                const float v8[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                store8<OUT>(a.Y, row * a.ld_out + chunk * 8, v8, k);
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

}  // namespace

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
