// Measurement aid: a kernel with the memory traffic of rq_rotate_quantize on 16-bit rows of width
// n = 512 T and no arithmetic to speak of.  One wave per row reads the row with the same 16-byte
// non-temporal loads (one kilobyte per load instruction) and writes n b / 8 bytes plus one float
// with the same non-temporal dword stores; the values written are an xor fold of the input, so
// nothing can be elided.  Its duration is the practical floor for a rotate_quantize launch of that
// shape: the benchmark reports it next to the real kernel.
#include "wave_common.h"

namespace rq {
namespace {

template <int BITS>
__global__ __launch_bounds__(64) void k_stream_reference(const uint16_t* X, int64_t rows, int t_loads, int64_t ld,
                                                         uint32_t* codes, float* scales) {
    const int lane = threadIdx.x;
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
        const uint16_t* xr = X + row * ld;
        uint32_t* out = codes + row * (int64_t)(t_loads * 16 * BITS);      // 512 T b / 32 dwords per row
        uint32_t all = 0;
        for (int t0 = 0; t0 < t_loads; t0 += 8) {
            u32x4 r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (t0 + u < t_loads) r[u] = load16(xr + ((t0 + u) * 64 + lane) * 8);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (t0 + u < t_loads) {
                    const uint32_t w = r[u][0] ^ r[u][1] ^ r[u][2] ^ r[u][3];
                    all ^= w;
                    const int group = (t0 + u) * 64 + lane;             // one group of 8 values
                    if (BITS == 4) store_codes(out + group, w);
                    else if ((group & 3) != 3) store_codes(out + (group >> 2) * 3 + (group & 3), w);
                }
        }
        if (lane == 0) scales[row] = __uint_as_float(all & 0x3fffffffu);
    }
}

}  // namespace

int stream_reference(const void* X, int64_t rows, int n, int64_t ld, int bits, uint32_t* codes, float* scales,
                     hipStream_t s) {
    const int64_t cap = 1 << 24;
    const dim3 grid((unsigned)(rows < cap ? rows : cap)), block(64);
    const uint16_t* x = static_cast<const uint16_t*>(X);
    if (bits == 4) hipLaunchKernelGGL(k_stream_reference<4>, grid, block, 0, s, x, rows, n / 512, ld, codes, scales);
    else hipLaunchKernelGGL(k_stream_reference<3>, grid, block, 0, s, x, rows, n / 512, ld, codes, scales);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace rq
