// General rotate-and-quantize kernels: one 256-thread workgroup per row, the row held in LDS.
// They cover every supported order p * 2^k that fits in LDS and all input types, and serve as
// the fallback for shapes the specialised wave kernels do not handle.
// The quantizing kernels hold the row as fp32 for 16-bit inputs and as fp64 for fp32 inputs: sums of
// 16-bit values lose next to nothing in fp32, but log2(n) fp32 butterfly stages on 24-bit inputs move a
// rotated value by up to ~2e-7 of its size, enough to push one in a million across a rounding
// boundary that the exact value misses by more than the 1e-6 the codes are allowed.
//
// Per row: load + zero-pad (section 4.2, Eq. 2) -> butterflies along the 2^k axis
// (section 2.3.2, Eq. 1) -> dense +-1 block product along the p axis (section 2.3.3) ->
// absmax -> scale -> round/clamp/pack (section 2.1 with the clip ratio of section 3.1).
#include "rotq_internal.h"

namespace rq {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxGroups = 320;      // groups of 128 in the longest row LDS can hold

__device__ __forceinline__ float load_f32(const void* X, int dtype, int64_t idx) {
    if (dtype == RQ_BF16) {
        uint32_t b = static_cast<const uint16_t*>(X)[idx];
        return __uint_as_float(b << 16);
    }
    if (dtype == RQ_F16) return (float)static_cast<const _Float16*>(X)[idx];      // exact
    return static_cast<const float*>(X)[idx];
}

__device__ __forceinline__ float wave_max(float v) {
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
    for (int m = 32; m >= 1; m >>= 1) v = fmax(v, __shfl_xor(v, m, 64));
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// Transforms the row held in buf0 (n floats, already visible to the whole workgroup) in place
// and returns the buffer that holds the un-normalised result H_n v, or H_n^T v when `transpose`
// is set ((H_p (x) H_m)^T = H_p^T (x) H_m: only the +-1 block changes).
template <typename T>
__device__ T* transform_row_lds(const RowArgs& a, T* buf0, T* buf1, bool transpose) {
    const int tid = threadIdx.x;
    const int n = a.n;
    for (int s = 0; s < a.log2m; ++s) {
        const int h = 1 << s;
        for (int idx = tid; idx < n / 2; idx += kThreads) {
            const int i = ((idx >> s) << (s + 1)) | (idx & (h - 1));
            const T u = buf0[i], v = buf0[i + h];
            buf0[i] = u + v;
            buf0[i + h] = u - v;
        }
        __syncthreads();
    }
    if (a.p == 1) return buf0;
    const int m = 1 << a.log2m;
    for (int o = tid; o < n; o += kThreads) {
        const int ao = o >> a.log2m, c = o & (m - 1);
        const int8_t* hrow = transpose ? a.block + ao : a.block + (size_t)ao * a.p;
        const int hstep = transpose ? a.p : 1;
        double acc = 0.0;
        for (int ai = 0; ai < a.p; ++ai) {
            const T v = buf0[ai * m + c];
            acc += (hrow[(size_t)ai * hstep] > 0) ? (double)v : -(double)v;
        }
        buf1[o] = (T)acc;
    }
    __syncthreads();
    return buf1;
}

template <typename T>
__device__ void load_row_lds(const RowArgs& a, int64_t row, T* buf0) {
    const int64_t base = row * a.ld;
    for (int j = threadIdx.x; j < a.n; j += kThreads)
        buf0[j] = (j < a.d) ? (T)load_f32(a.X, a.dtype, base + j) : (T)0;
    __syncthreads();
}

// Rotates one row into LDS (un-normalised: y_u = H_n pad(x)) and returns the buffer that holds
// it; also returns the row's max |y_u| in *amax (same value in every thread).
template <typename T>
__device__ T* rotate_row_lds(const RowArgs& a, int64_t row, T* buf0, T* buf1, T* red, T* amax) {
    const int tid = threadIdx.x;
    const int n = a.n;
    load_row_lds(a, row, buf0);
    T* y = transform_row_lds(a, buf0, buf1, false);
    T mx = 0;
    for (int j = tid; j < n; j += kThreads) {
        const T v = y[j];
        const T av = v < 0 ? -v : v;
        mx = av > mx ? av : mx;
    }
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    T r = red[0];
    for (int w = 1; w < 4; ++w) r = red[w] > r ? red[w] : r;
    *amax = r;
    return y;
}

__device__ __forceinline__ float round_clamp(float t, float lo, float hi) { return fminf(fmaxf(rintf(t), lo), hi); }
__device__ __forceinline__ double round_clamp(double t, double lo, double hi) { return fmin(fmax(rint(t), lo), hi); }

// Store of one result value as fp32 or bf16 (round to nearest even).
__device__ __forceinline__ void store_out(const OutArgs& o, int64_t idx, float v) {
    if (o.dtype == RQ_BF16) {
        const uint32_t u = __float_as_uint(v);
        static_cast<uint16_t*>(o.Y)[idx] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    } else if (o.dtype == RQ_F16) {
        static_cast<_Float16*>(o.Y)[idx] = (_Float16)v;
    } else {
        static_cast<float*>(o.Y)[idx] = v;
    }
}

// Rotation alone, floating-point result: Y = (H_n pad(x) / sqrt(n))[:d_out], or with H_n^T.
// Serves the offline weight fusion of section 4.2 (Eq. 2: rows of W^T or of W) and the
// inverse rotation x = H_n^T y / sqrt(n) (section 2.3).
__global__ __launch_bounds__(kThreads) void k_generic_rotate(RowArgs a, int transpose, OutArgs o) {
    extern __shared__ float lds[];
    const int64_t row = blockIdx.x;
    load_row_lds(a, row, lds);
    const float* y = transform_row_lds(a, lds, lds + a.n, transpose != 0);
    const double inv = 1.0 / sqrt((double)a.n);
    for (int j = threadIdx.x; j < o.d_out; j += kThreads)
        store_out(o, row * o.ld_out + j, (float)((double)y[j] * inv));
}

// Dequantize-and-rotate-back: y^ from packed codes (symmetric: code * Delta, the transform then
// runs on the integer codes, which fp32 adds exactly; asymmetric groups of 128: code * Delta_g +
// lo_g), then H_n^T y^ / sqrt(n), first d_out columns.
__global__ __launch_bounds__(kThreads) void k_generic_dequant_rotate(RowArgs a, const uint32_t* codes,
                                                                     const float* scales,
                                                                     const float* mins, int transpose,
                                                                     OutArgs o) {
    extern __shared__ float lds[];
    const int64_t row = blockIdx.x;
    const int bits = a.bits;
    const uint8_t* cr = reinterpret_cast<const uint8_t*>(codes) + row * (int64_t)(a.n / 8 * bits);
    const uint32_t mask = (1u << bits) - 1u;
    const int n_groups = a.n / 128;
    for (int j = threadIdx.x; j < a.n; j += kThreads) {
        const int bit = j * bits, by = bit >> 3, sh = bit & 7;
        uint32_t w = cr[by];
        if (sh + bits > 8) w |= (uint32_t)cr[by + 1] << 8;         // never beyond the row's last byte
        const uint32_t f = (w >> sh) & mask;
        if (mins) {
            const int64_t gi = row * n_groups + (j >> 7);
            lds[j] = fmaf((float)f, scales[gi], mins[gi]);
        } else {
            lds[j] = (float)((int)(f << (32 - bits)) >> (32 - bits));
        }
    }
    __syncthreads();
    const float* y = transform_row_lds(a, lds, lds + a.n, transpose != 0);
    const double k = (mins ? 1.0 : (double)scales[row]) / sqrt((double)a.n);
    for (int j = threadIdx.x; j < o.d_out; j += kThreads)
        store_out(o, row * o.ld_out + j, (float)((double)y[j] * k));
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_generic_rotate_quantize(RowArgs a, float clip,
                                                                      uint32_t* codes,
                                                                      float* scales) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_bytes_[];
    T* const lds = reinterpret_cast<T*>(lds_bytes_);
    __shared__ T red[4];
    const int64_t row = blockIdx.x;
    T amax;
    const T* y = rotate_row_lds<T>(a, row, lds, lds + a.n, red, &amax);
    const int bits = a.bits;
    const double lvl = (double)((1 << bits) - 1);
    const T qmax = (T)((1 << (bits - 1)) - 1), qmin = -(T)(1 << (bits - 1));
    // fp32 rows: one rounding of lvl / (clip amax); fp64 rows: the quotient itself
    const T s = amax > 0 ? (T)(lvl / ((double)clip * (double)amax)) : (T)0;
    if (threadIdx.x == 0)
        scales[row] = (float)((double)clip * (double)amax / (sqrt((double)a.n) * lvl));
    const uint32_t mask = (1u << bits) - 1u;
    if (a.n % 32 != 0) {
        // orders that are only a multiple of 8 (whole-dimension blocks such as 1544): a row is a whole
        // number of bytes but not of dwords, so groups of 8 codes are stored byte by byte
        uint8_t* outb = reinterpret_cast<uint8_t*>(codes) + row * (int64_t)(a.n / 8 * bits);
        for (int g = threadIdx.x; g < a.n / 8; g += kThreads) {
            uint32_t acc = 0;
            for (int e = 0; e < 8; ++e) {
                const T t = y[g * 8 + e] * s;
                const int q = (int)round_clamp(t, qmin, qmax);
                acc |= ((uint32_t)q & mask) << (e * bits);
            }
            for (int k = 0; k < bits; ++k) outb[g * bits + k] = (uint8_t)(acc >> (8 * k));
        }
        return;
    }
    uint32_t* out = codes + row * (int64_t)(a.n / 32 * bits);
    for (int g = threadIdx.x; g < a.n / 32; g += kThreads) {
        uint64_t acc = 0;
        int nb = 0, w = 0;
        for (int e = 0; e < 32; ++e) {
            const T t = y[g * 32 + e] * s;
            const int q = (int)round_clamp(t, qmin, qmax);
            acc |= (uint64_t)((uint32_t)q & mask) << nb;
            nb += bits;
            if (nb >= 32) {
                out[g * bits + w++] = (uint32_t)acc;
                acc >>= 32;
                nb -= 32;
            }
        }
    }
}

// Asymmetric quantization in groups of 128 rotated values (section 5.1, KV cache): per group
// lo = clip * min, delta = clip * (max - min) / (2^b - 1), code = clamp(rne((y - lo) / delta), 0,
// 2^b - 1).  The decision is taken in fp64 here; this kernel is the general fallback.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_generic_rotate_quantize_asym(RowArgs a, float clip,
                                                                           uint32_t* codes,
                                                                           float* scales, float* mins) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_bytes_[];
    T* const lds = reinterpret_cast<T*>(lds_bytes_);
    __shared__ T red[4];
    __shared__ T gmn[kMaxGroups], gmx[kMaxGroups];
    const int64_t row = blockIdx.x;
    T amax;
    const T* y = rotate_row_lds<T>(a, row, lds, lds + a.n, red, &amax);
    const int bits = a.bits;
    const int n_groups = a.n / 128;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int gi = wave; gi < n_groups; gi += kThreads / 64) {
        const T u = y[gi * 128 + lane], v = y[gi * 128 + 64 + lane];
        T mn = u < v ? u : v, mx = u < v ? v : u;
        for (int m = 32; m >= 1; m >>= 1) {
            const T on = __shfl_xor(mn, m, 64), ox = __shfl_xor(mx, m, 64);
            mn = on < mn ? on : mn;
            mx = ox > mx ? ox : mx;
        }
        if (lane == 0) {
            gmn[gi] = mn;
            gmx[gi] = mx;
        }
    }
    __syncthreads();
    const double lvl = (double)((1 << bits) - 1);
    const double rn = sqrt((double)a.n);
    for (int gi = threadIdx.x; gi < n_groups; gi += kThreads) {
        const double r = (double)gmx[gi] - (double)gmn[gi];
        scales[row * n_groups + gi] = (float)((double)clip * r / (rn * lvl));
        mins[row * n_groups + gi] = (float)((double)clip * (double)gmn[gi] / rn);
    }
    const uint32_t mask = (1u << bits) - 1u;
    uint32_t* out = codes + row * (int64_t)(a.n / 32 * bits);
    for (int g = threadIdx.x; g < a.n / 32; g += kThreads) {
        const double mn = (double)gmn[g >> 2];
        const double r = (double)gmx[g >> 2] - mn;
        const double lo = (double)clip * mn;
        const double inv = r > 0.0 ? lvl / ((double)clip * r) : 0.0;
        uint64_t acc = 0;
        int nb = 0, w = 0;
        for (int e = 0; e < 32; ++e) {
            const double t = ((double)y[g * 32 + e] - lo) * inv;
            const int q = (int)fmin(fmax(rint(t), 0.0), lvl);
            acc |= (uint64_t)((uint32_t)q & mask) << nb;
            nb += bits;
            if (nb >= 32) {
                out[g * bits + w++] = (uint32_t)acc;
                acc >>= 32;
                nb -= 32;
            }
        }
    }
}

// Per-token symmetric quantization of rows as they are (section 2.1; no rotation, for layers
// whose rotation is fused into the weights).  One workgroup per row, two passes over the row:
// absmax, then round / clamp / pack (the second pass is served by the caches).
__global__ __launch_bounds__(kThreads) void k_plain_quantize(const void* X, int dtype, int d, int64_t ld,
                                                             int bits, float clip, uint32_t* codes,
                                                             float* scales) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const int64_t base = row * ld;
    float mx = 0.0f;
    for (int j = threadIdx.x; j < d; j += kThreads) mx = fmaxf(mx, fabsf(load_f32(X, dtype, base + j)));
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    const float amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const double lvl = (double)((1 << bits) - 1);
    const float qmax = (float)((1 << (bits - 1)) - 1), qmin = -(float)(1 << (bits - 1));
    const float s = amax > 0.0f ? (float)(lvl / ((double)clip * (double)amax)) : 0.0f;
    const double delta = (double)clip * (double)amax / lvl;
    if (threadIdx.x == 0) scales[row] = (float)delta;
    const uint32_t mask = (1u << bits) - 1u;
    uint32_t* out = codes + row * (int64_t)(d / 32 * bits);
    for (int g = threadIdx.x; g < d / 32; g += kThreads) {
        uint64_t acc = 0;
        int nb = 0, w = 0;
        for (int e = 0; e < 32; ++e) {
            const float x = load_f32(X, dtype, base + g * 32 + e);
            const float t = x * s;
            float r = rintf(t);
            // un-rotated bf16 inputs sit on a coarse grid and hit rounding ties often: near a tie
            // the decision is retaken with the exact quotient x / Delta in fp64
            if (fabsf(t - r) > 0.499f) r = (float)rint((double)x / delta);
            const int q = (int)fminf(fmaxf(r, qmin), qmax);
            acc |= (uint64_t)((uint32_t)q & mask) << nb;
            nb += bits;
            if (nb >= 32) {
                out[g * bits + w++] = (uint32_t)acc;
                acc >>= 32;
                nb -= 32;
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_generic_quant_error(RowArgs a, ClipList clips,
                                                                  int n_clips, double* partial) {
    extern __shared__ float lds[];
    __shared__ float red[4];
    __shared__ double dred[4];
    const int64_t row = blockIdx.x;
    float amax;
    const float* y = rotate_row_lds(a, row, lds, lds + a.n, red, &amax);
    const int bits = a.bits;
    const double lvl = (double)((1 << bits) - 1);
    const float qmax = (float)((1 << (bits - 1)) - 1), qmin = -(float)(1 << (bits - 1));
    for (int k = 0; k < n_clips; ++k) {
        const double dk64 = (double)clips.v[k] * (double)amax / lvl;
        const float dk = (float)dk64;
        const float ik = amax > 0.0f ? (float)(1.0 / dk64) : 0.0f;
        float acc = 0.0f;
        for (int j = threadIdx.x; j < a.n; j += kThreads) {
            const float v = y[j];
            const float q = fminf(fmaxf(rintf(v * ik), qmin), qmax);
            const float e = fmaf(-q, dk, v);
            acc = fmaf(e, e, acc);
        }
        double tot = wave_sum((double)acc);
        if ((threadIdx.x & 63) == 0) dred[threadIdx.x >> 6] = tot;
        __syncthreads();
        if (threadIdx.x == 0)
            partial[row * n_clips + k] =
                (dred[0] + dred[1] + dred[2] + dred[3]) / ((double)a.n * (double)a.n);
        __syncthreads();
    }
}

// quant_error with the asymmetric group-128 quantizer (sections 4.1, 5.1): per group lo = clip min,
// Delta = clip (max - min) / (2^b - 1); e = y - (code Delta + lo).
__global__ __launch_bounds__(kThreads) void k_generic_quant_error_asym(RowArgs a, ClipList clips,
                                                                       int n_clips, double* partial) {
    extern __shared__ float lds[];
    __shared__ float red[4];
    __shared__ double dred[4];
    __shared__ float gmn[kMaxGroups], gmx[kMaxGroups];
    const int64_t row = blockIdx.x;
    float amax;
    const float* y = rotate_row_lds(a, row, lds, lds + a.n, red, &amax);
    const int n_groups = a.n / 128;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int gi = wave; gi < n_groups; gi += kThreads / 64) {
        const float u = y[gi * 128 + lane], v = y[gi * 128 + 64 + lane];
        float mn = fminf(u, v), mx = fmaxf(u, v);
        for (int m = 32; m >= 1; m >>= 1) {
            mn = fminf(mn, __shfl_xor(mn, m, 64));
            mx = fmaxf(mx, __shfl_xor(mx, m, 64));
        }
        if (lane == 0) {
            gmn[gi] = mn;
            gmx[gi] = mx;
        }
    }
    __syncthreads();
    const double lvl = (double)((1 << a.bits) - 1);
    for (int k = 0; k < n_clips; ++k) {
        const double cl = (double)clips.v[k];
        float acc = 0.0f;
        for (int j = threadIdx.x; j < a.n; j += kThreads) {
            const double mn = (double)gmn[j >> 7], r = (double)gmx[j >> 7] - mn;
            const float lo = (float)(cl * mn), dk = (float)(cl * r / lvl);
            const float ik = r > 0.0 ? (float)(lvl / (cl * r)) : 0.0f;
            const float d = y[j] - lo;
            const float q = fminf(fmaxf(rintf(d * ik), 0.0f), (float)lvl);
            const float e = fmaf(-q, dk, d);
            acc = fmaf(e, e, acc);
        }
        double tot = wave_sum((double)acc);
        if ((threadIdx.x & 63) == 0) dred[threadIdx.x >> 6] = tot;
        __syncthreads();
        if (threadIdx.x == 0)
            partial[row * n_clips + k] =
                (dred[0] + dred[1] + dred[2] + dred[3]) / ((double)a.n * (double)a.n);
        __syncthreads();
    }
}

// partial[row][k] is the row's mean squared error in the normalised domain (un-normalised sum
// divided by n twice); mse[k] is its mean over rows, summed in a fixed order.
__global__ __launch_bounds__(kThreads) void k_reduce_partials(const double* partial, int64_t count,
                                                              int64_t stride, int64_t rows, int n_clips,
                                                              float* mse) {
    // sums partial[(i * stride)][k], i < count, in a fixed order; mse[k] = sum / rows
    __shared__ double dred[4];
    const int k = blockIdx.x;
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += kThreads) acc += partial[i * stride * n_clips + k];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) dred[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0)
        mse[k] = rows > 0 ? (float)((dred[0] + dred[1] + dred[2] + dred[3]) / (double)rows) : 0.0f;
}

// First level for many rows: one workgroup sums a chunk of kChunkRows rows for every clip ratio
// (coalesced: consecutive threads read consecutive clip ratios of a row) and leaves the sums in the
// chunk's own first row - read by no other workgroup - so no extra workspace is needed.
constexpr int kChunkRows = 256;

__global__ __launch_bounds__(kThreads) void k_reduce_chunks(double* partial, int64_t rows, int n_clips) {
    __shared__ double part[kThreads];
    int kp = 1;
    while (kp < n_clips) kp <<= 1;                       // n_clips <= 64
    const int lanes = kThreads / kp;                     // row lanes
    const int k = threadIdx.x % kp, rl = threadIdx.x / kp;
    const int64_t row0 = (int64_t)blockIdx.x * kChunkRows;
    const int64_t left = rows - row0;
    const int nrows = left < kChunkRows ? (int)left : kChunkRows;
    double acc = 0.0;
    if (k < n_clips)
        for (int r = rl; r < nrows; r += lanes) acc += partial[(row0 + r) * n_clips + k];
    part[threadIdx.x] = acc;
    __syncthreads();                                     // every read of the chunk is done
    if (rl == 0 && k < n_clips) {
        double t = 0.0;
        for (int i = 0; i < lanes; ++i) t += part[i * kp + k];
        partial[row0 * n_clips + k] = t;
    }
}

size_t lds_bytes(const rq_hadamard* h) {
    return (size_t)h->f.n * sizeof(float) * (h->f.p > 1 ? 2 : 1);
}

template <typename K>
int prepare(K kernel, size_t bytes) {
    if (bytes > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return RQ_ERR_HIP;
    }
    return RQ_OK;
}

}  // namespace

bool generic_supports(const rq_hadamard* h) { return h->device >= 0 && h->generic_ok; }

// Called once when the handle is built (never on the hot path): checks that the row fits in
// LDS and raises the kernels' dynamic-LDS limit where the default does not cover it.
bool generic_prepare(rq_hadamard* h) {
    const size_t bytes = lds_bytes(h);
    h->generic_f64_ok = false;
    if (bytes + 256 > (size_t)h->max_lds) return false;
    if (h->f.n % 128 == 0 && (h->f.n / 128 > kMaxGroups ||
                              prepare(k_generic_rotate_quantize_asym<float>, bytes) != RQ_OK))
        return false;
    if (prepare(k_generic_rotate, bytes) != RQ_OK || prepare(k_generic_dequant_rotate, bytes) != RQ_OK)
        return false;
    if (h->f.n % 128 == 0 && prepare(k_generic_quant_error_asym, bytes) != RQ_OK) return false;
    if (prepare(k_generic_rotate_quantize<float>, bytes) != RQ_OK || prepare(k_generic_quant_error, bytes) != RQ_OK)
        return false;
    // fp32 rows are quantized from an fp64 copy of the row: twice the LDS (plus the fp64 group extremes)
    h->generic_f64_ok = 2 * bytes + 8 * 1024 <= (size_t)h->max_lds &&
                        prepare(k_generic_rotate_quantize<double>, 2 * bytes) == RQ_OK &&
                        (h->f.n % 128 != 0 || prepare(k_generic_rotate_quantize_asym<double>, 2 * bytes) == RQ_OK);
    return true;
}

int generic_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                            float* scales, hipStream_t s) {
    const size_t bytes = lds_bytes(h);
    if (a.rows > 0x7fffffffLL) return RQ_ERR_ARG;
    if (a.dtype == RQ_F32) {
        if (!h->generic_f64_ok) return RQ_ERR_NO_ORDER;
        hipLaunchKernelGGL(k_generic_rotate_quantize<double>, dim3((unsigned)a.rows), dim3(kThreads), 2 * bytes,
                           s, a, clip, codes, scales);
    } else {
        hipLaunchKernelGGL(k_generic_rotate_quantize<float>, dim3((unsigned)a.rows), dim3(kThreads), bytes, s, a,
                           clip, codes, scales);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int generic_rotate_quantize_asym(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                                 float* scales, float* mins, hipStream_t s) {
    const size_t bytes = lds_bytes(h);
    if (a.rows > 0x7fffffffLL || a.n % 128 != 0) return RQ_ERR_ARG;
    if (a.dtype == RQ_F32) {
        if (!h->generic_f64_ok) return RQ_ERR_NO_ORDER;
        hipLaunchKernelGGL(k_generic_rotate_quantize_asym<double>, dim3((unsigned)a.rows), dim3(kThreads),
                           2 * bytes, s, a, clip, codes, scales, mins);
    } else {
        hipLaunchKernelGGL(k_generic_rotate_quantize_asym<float>, dim3((unsigned)a.rows), dim3(kThreads), bytes,
                           s, a, clip, codes, scales, mins);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int generic_rotate(const rq_hadamard* h, const RowArgs& a, int transpose, const OutArgs& o,
                   hipStream_t s) {
    if (a.rows > 0x7fffffffLL) return RQ_ERR_ARG;
    hipLaunchKernelGGL(k_generic_rotate, dim3((unsigned)a.rows), dim3(kThreads), lds_bytes(h), s, a,
                       transpose, o);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int generic_dequant_rotate(const rq_hadamard* h, const RowArgs& a, const uint32_t* codes,
                           const float* scales, const float* mins, int transpose, const OutArgs& o,
                           hipStream_t s) {
    if (a.rows > 0x7fffffffLL) return RQ_ERR_ARG;
    hipLaunchKernelGGL(k_generic_dequant_rotate, dim3((unsigned)a.rows), dim3(kThreads), lds_bytes(h), s,
                       a, codes, scales, mins, transpose, o);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int plain_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                   uint32_t* codes, float* scales, hipStream_t s) {
    if (rows > 0x7fffffffLL) return RQ_ERR_ARG;
    hipLaunchKernelGGL(k_plain_quantize, dim3((unsigned)rows), dim3(kThreads), 0, s, X, dtype, d, ld,
                       bits, clip, codes, scales);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int reduce_partials(double* partial, int64_t rows, int n_clips, float* mse, hipStream_t s) {
    if (rows > 16 * kChunkRows) {
        const int64_t chunks = (rows + kChunkRows - 1) / kChunkRows;
        if (chunks > 0x7fffffffLL) return RQ_ERR_ARG;
        hipLaunchKernelGGL(k_reduce_chunks, dim3((unsigned)chunks), dim3(kThreads), 0, s, partial, rows, n_clips);
        hipLaunchKernelGGL(k_reduce_partials, dim3(n_clips), dim3(kThreads), 0, s, partial, chunks,
                           (int64_t)kChunkRows, rows, n_clips, mse);
    } else {
        hipLaunchKernelGGL(k_reduce_partials, dim3(n_clips), dim3(kThreads), 0, s, partial, rows, (int64_t)1,
                           rows, n_clips, mse);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int generic_quant_error_asym(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                             float* mse, double* partial, hipStream_t s) {
    const size_t bytes = lds_bytes(h);
    if (a.rows > 0x7fffffffLL || a.n % 128 != 0) return RQ_ERR_ARG;
    if (a.rows > 0) {
        hipLaunchKernelGGL(k_generic_quant_error_asym, dim3((unsigned)a.rows), dim3(kThreads), bytes, s, a,
                           clips, n_clips, partial);
        if (hipGetLastError() != hipSuccess) return RQ_ERR_HIP;
    }
    return reduce_partials(partial, a.rows, n_clips, mse, s);
}

int generic_quant_error(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                        float* mse, double* partial, hipStream_t s) {
    const size_t bytes = lds_bytes(h);
    if (a.rows > 0x7fffffffLL) return RQ_ERR_ARG;
    if (a.rows > 0) {
        hipLaunchKernelGGL(k_generic_quant_error, dim3((unsigned)a.rows), dim3(kThreads), bytes, s, a,
                           clips, n_clips, partial);
        if (hipGetLastError() != hipSuccess) return RQ_ERR_HIP;
    }
    return reduce_partials(partial, a.rows, n_clips, mse, s);
}

}  // namespace rq
