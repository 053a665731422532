// Dequantizer in the rotated domain (section 2.1: X^ = round(X / Delta) * Delta): packed b-bit codes
// and their scales back to floating-point values, without a rotation.  y^_j = code_j * Delta for the
// signed per-token codes, code_j * Delta_g + lo_g for the unsigned group-128 codes (section 5.1).
// One thread takes 4 codes (2 bytes of the row's bit stream for b = 4, 12 bits for b = 3) and writes
// one 16-byte unit, so a store instruction of a wave covers 1 KB of consecutive output - the kernel
// is all stores (16 bytes out per 1.5 - 2 bytes in).  Rows shorter than a workgroup share one:
// a workgroup of 256 threads takes floor(1024 / n) whole rows; longer rows are cut into segments of
// 1024 values along grid.x.  All index arithmetic is 32-bit; the row of a thread inside its
// workgroup is a multiply-high with ceil(2^32 / (n / 4)), exact for the values below 256 it sees.
#include "rotq_internal.h"

namespace rq {
namespace {

constexpr int kThreads = 256;
// Row groups a thread takes per iteration (their loads go out together).  Measured: 1 is best where it matters
// (4096-wide rows 0.95 of the HBM peak against 0.89 with 4, head rows of 128 with 3-bit codes 0.87 against 0.79);
// only 4-bit head rows gain from 4 (0.59 -> 0.70).
constexpr int kGroupsPerIteration = 1;

template <int BITS, bool ASYM>
__global__ __launch_bounds__(kThreads) void k_dequantize(const uint8_t* codes, const float* scales,
                                                         const float* mins, int64_t rows, int n, uint32_t qpr_magic,
                                                         int rows_per_group, float* Y, bool y16) {
    const int qpr = n >> 2;                                  // 4-value units per row
    int r_local = 0, q = (int)(blockIdx.x * kThreads + threadIdx.x);
    if (rows_per_group > 1) {                                // short rows: several per workgroup, grid.x == 1
        r_local = (int)__umulhi(threadIdx.x, qpr_magic);
        q = (int)threadIdx.x - r_local * qpr;
        if (r_local >= rows_per_group) return;
    } else if (q >= qpr) {
        return;
    }
    const int row_bytes = n * BITS / 8;
    constexpr int U = kGroupsPerIteration;
    for (int64_t grp0 = (int64_t)blockIdx.y * U; grp0 * rows_per_group < rows; grp0 += (int64_t)gridDim.y * U) {
        uint32_t w[U];
        float delta[U], lo[U];
        int64_t row[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            row[u] = (grp0 + u) * rows_per_group + r_local;
            const int64_t rl = row[u] < rows ? row[u] : rows - 1;            // rows beyond the end: loads only
            const uint8_t* p = codes + rl * row_bytes;
            if constexpr (BITS == 4) {
                w[u] = *reinterpret_cast<const uint16_t*>(p + 2 * q);       // rows are whole dwords: 2-byte aligned
            } else {
                const int byte = (3 * q) >> 1;                               // 12 q bits in
                w[u] = ((uint32_t)p[byte] | ((uint32_t)p[byte + 1] << 8)) >> (4 * (q & 1));
            }
            lo[u] = 0.0f;
            if constexpr (ASYM) {
                const int64_t gi = rl * (n / RQ_GROUP) + (4 * q) / RQ_GROUP;
                delta[u] = scales[gi];
                lo[u] = mins[gi];
            } else {
                delta[u] = scales[rl];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (row[u] >= rows) break;
            float v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t f = (w[u] >> (BITS * k)) & ((1u << BITS) - 1u);
                if constexpr (ASYM) {
                    v[k] = fmaf((float)f, delta[u], lo[u]);
                } else {
                    const int c = (int)(f ^ (1u << (BITS - 1))) - (1 << (BITS - 1));   // two's complement field
                    v[k] = (float)c * delta[u];
                }
            }
            float* out = Y + row[u] * (int64_t)n + 4 * q;
            if (y16) {
                typedef float f32x4_t __attribute__((ext_vector_type(4)));
                __builtin_nontemporal_store(f32x4_t{v[0], v[1], v[2], v[3]}, reinterpret_cast<f32x4_t*>(out));
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) out[k] = v[k];
            }
        }
    }
}

}  // namespace

int dequantize_rows(const uint32_t* codes, const float* scales, const float* mins, int64_t rows, int n, int bits,
                    float* Y, hipStream_t s) {
    const int qpr = n >> 2;                                          // n is a multiple of 8
    const int rows_per_group = qpr >= kThreads ? 1 : kThreads / qpr;
    const uint32_t magic = (uint32_t)((0x100000000ull + (uint64_t)qpr - 1) / (uint64_t)qpr);
    const int64_t groups = (rows + rows_per_group - 1) / rows_per_group;
    const int64_t quads = (groups + kGroupsPerIteration - 1) / kGroupsPerIteration;
    const dim3 grid(rows_per_group > 1 ? 1u : (unsigned)((qpr + kThreads - 1) / kThreads),
                    (unsigned)(quads < 65535 ? quads : 65535));
    const bool y16 = (reinterpret_cast<uintptr_t>(Y) & 15) == 0;     // rows are n * 4 bytes, n a multiple of 8
    const uint8_t* c = reinterpret_cast<const uint8_t*>(codes);
    if (mins) {
        if (bits == 4) hipLaunchKernelGGL((k_dequantize<4, true>), grid, dim3(kThreads), 0, s, c, scales, mins, rows, n, magic, rows_per_group, Y, y16);
        else hipLaunchKernelGGL((k_dequantize<3, true>), grid, dim3(kThreads), 0, s, c, scales, mins, rows, n, magic, rows_per_group, Y, y16);
    } else {
        if (bits == 4) hipLaunchKernelGGL((k_dequantize<4, false>), grid, dim3(kThreads), 0, s, c, scales, mins, rows, n, magic, rows_per_group, Y, y16);
        else hipLaunchKernelGGL((k_dequantize<3, false>), grid, dim3(kThreads), 0, s, c, scales, mins, rows, n, magic, rows_per_group, Y, y16);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace rq
