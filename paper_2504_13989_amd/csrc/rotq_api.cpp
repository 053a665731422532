// C ABI: argument validation, handle management and kernel dispatch.
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "rotq_internal.h"

namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_rows(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
               int bits) {
    if (!h) return RQ_ERR_ARG;
    if (dtype != RQ_BF16 && dtype != RQ_F32 && dtype != RQ_F16) return RQ_ERR_ARG;
    if (rows < 0 || d < 1 || d > h->f.n || ld < d) return RQ_ERR_ARG;
    if (bits != 3 && bits != 4) return RQ_ERR_ARG;
    // with no rows nothing is read or written through X / codes / scales: they may be NULL
    if (rows > 0 && (!X || !aligned(X, dtype == RQ_F32 ? 4 : 2))) return RQ_ERR_ARG;
    return RQ_OK;
}

bool clip_ok(float c) { return c > 0.0f && c <= 1.0f; }   // false for NaN

// records which kernel family a call chose (diagnostic; the handle's only field written after build)
void note(const rq_hadamard_t* h, const char* name) { h->last_kernel.store(name, std::memory_order_relaxed); }

rq::RowArgs row_args(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d,
                     int64_t ld, int bits) {
    return rq::RowArgs{X, dtype, rows, d, ld, h->f.n, h->f.p, h->f.log2m, h->d_block, bits};
}

}  // namespace

extern "C" {

int rq_hadamard_build(int n, rq_hadamard_t** out) {
    if (!out || n < 32) return RQ_ERR_ARG;
    if (n % 8 != 0) return RQ_ERR_NO_ORDER;     // packed rows are whole bytes for 3 and 4 bits
    rq::Factorisation f;
    if (!rq::factor_order(n, &f)) return RQ_ERR_NO_ORDER;
    rq_hadamard* h = new (std::nothrow) rq_hadamard;
    if (!h) return RQ_ERR_NOMEM;
    h->f = f;
    try {
        h->block = rq::build_block(f);
    } catch (const std::bad_alloc&) {
        delete h;
        return RQ_ERR_NOMEM;
    }
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count == 0) {
        (void)hipGetLastError();
        *out = h;   // host-only handle
        return RQ_OK;
    }
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        delete h;
        return RQ_ERR_HIP;
    }
    h->max_lds = (int)prop.sharedMemPerBlock;
    h->num_cu = prop.multiProcessorCount;
    const size_t bytes = h->block.size();
    if (hipMalloc((void**)&h->d_block, bytes) != hipSuccess ||
        hipMemcpy(h->d_block, h->block.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
        if (h->d_block) (void)hipFree(h->d_block);
        delete h;
        return RQ_ERR_HIP;
    }
    const bool sylv = f.p == 1 && f.log2m >= 7 && f.log2m <= 13;
    // block orders of the block kernels; the Sylvester orders 2^14, 2^15 ride along with p = 1
    const bool blk = (f.p > 1 && f.log2m >= 7 && (f.p << (f.log2m - 7)) <= 256) ||
                     (f.p == 1 && (f.log2m == 14 || f.log2m == 15));
    const bool blk_short = f.p > 1 && (f.log2m == 5 || f.log2m == 6) && f.p <= 256;   // block rows of 32 / 64
    const bool dense = !sylv && !blk && !blk_short && n <= 4096;
    if (sylv || blk || blk_short || dense) {
        std::vector<uint32_t> tiles;
        bool f16_table = sylv;
        if (sylv) {
            tiles = rq::wave_sylvester_tiles();
        } else if (dense) {
            std::vector<int8_t> hm((size_t)n * n);
            if (rq_hadamard_dense(h, hm.data()) != RQ_OK) {
                rq_hadamard_free(h);
                return RQ_ERR_ARG;
            }
            tiles = rq::dense_block_tiles(hm, n);
            h->dense_ok = true;
        } else if (blk_short) {
            tiles = rq::wg_block_tiles(h->block, f.p);
            h->wg_ok = rq::wg_block_prepare(f.p);
            f16_table = true;
        } else {
            // block of the strided axis: H_p (x) H_{2^(k-7)}, index a * 2^(k-7) + (high bits of c)
            const int e = 1 << (f.log2m - 7), pb = f.p * e;
            std::vector<int8_t> bm((size_t)pb * pb);
            for (int i = 0; i < pb; ++i)
                for (int j = 0; j < pb; ++j)
                    bm[(size_t)i * pb + j] = (int8_t)(h->block[(size_t)(i / e) * f.p + j / e] *
                                                      rq::sylvester_entry(i % e, j % e));
            tiles = pb <= 32 ? rq::wave_block_tiles(bm, pb) : rq::wg_block_tiles(bm, pb);
            if (pb > 32) h->wg_ok = rq::wg_block_prepare(pb);
            f16_table = true;
            if (pb <= 32) {
                // the transposed block's tiles: rq_rotate with transpose = 1 (Paley I blocks are not symmetric)
                std::vector<int8_t> bt((size_t)pb * pb);
                for (int i = 0; i < pb; ++i)
                    for (int j = 0; j < pb; ++j) bt[(size_t)i * pb + j] = bm[(size_t)j * pb + i];
                const std::vector<uint32_t> tt = rq::wave_block_tiles(bt, pb), tth = rq::tiles_to_f16(tt);
                const size_t bb = tt.size() * sizeof(uint32_t);
                if (hipMalloc(&h->d_tiles_t, bb) != hipSuccess || hipMalloc(&h->d_tiles_t_f16, bb) != hipSuccess ||
                    hipMemcpy(h->d_tiles_t, tt.data(), bb, hipMemcpyHostToDevice) != hipSuccess ||
                    hipMemcpy(h->d_tiles_t_f16, tth.data(), bb, hipMemcpyHostToDevice) != hipSuccess) {
                    rq_hadamard_free(h);
                    return RQ_ERR_HIP;
                }
            }
            if (pb > 32 && pb <= 64) {
                // these blocks also have a one-wave kernel (rotate_quantize), with operand tiles of its own
                const std::vector<uint32_t> t2 = rq::wave_block2_tiles(bm, pb), t2h = rq::tiles_to_f16(t2);
                const size_t b2 = t2.size() * sizeof(uint32_t);
                if (hipMalloc(&h->d_tiles2, b2) != hipSuccess || hipMalloc(&h->d_tiles2_f16, b2) != hipSuccess ||
                    hipMemcpy(h->d_tiles2, t2.data(), b2, hipMemcpyHostToDevice) != hipSuccess ||
                    hipMemcpy(h->d_tiles2_f16, t2h.data(), b2, hipMemcpyHostToDevice) != hipSuccess) {
                    rq_hadamard_free(h);
                    return RQ_ERR_HIP;
                }
            }
        }
        const size_t tb = tiles.size() * sizeof(uint32_t);
        if (hipMalloc(&h->d_tiles, tb) != hipSuccess ||
            hipMemcpy(h->d_tiles, tiles.data(), tb, hipMemcpyHostToDevice) != hipSuccess) {
            rq_hadamard_free(h);
            return RQ_ERR_HIP;
        }
        if (f16_table) {
            const std::vector<uint32_t> t16 = rq::tiles_to_f16(tiles);
            if (hipMalloc(&h->d_tiles_f16, tb) != hipSuccess ||
                hipMemcpy(h->d_tiles_f16, t16.data(), tb, hipMemcpyHostToDevice) != hipSuccess) {
                rq_hadamard_free(h);
                return RQ_ERR_HIP;
            }
        }
    }
    h->device = dev;
    h->generic_ok = rq::generic_prepare(h);
    // set-up time is when the static scratch array's address on this device is asked for; a failure
    // only makes rq_quant_error_noalloc return RQ_ERR_HIP
    (void)rq::static_scratch(dev);
    *out = h;
    return RQ_OK;
}

void rq_hadamard_free(rq_hadamard_t* h) {
    if (!h) return;
    if (h->d_block) (void)hipFree(h->d_block);
    if (h->d_tiles) (void)hipFree(h->d_tiles);
    if (h->d_tiles_f16) (void)hipFree(h->d_tiles_f16);
    if (h->d_tiles_t) (void)hipFree(h->d_tiles_t);
    if (h->d_tiles_t_f16) (void)hipFree(h->d_tiles_t_f16);
    if (h->d_tiles2) (void)hipFree(h->d_tiles2);
    if (h->d_tiles2_f16) (void)hipFree(h->d_tiles2_f16);
    delete h;
}

int rq_hadamard_info(const rq_hadamard_t* h, int* n, int* p, int* kind, int* q, int* log2m) {
    if (!h) return RQ_ERR_ARG;
    if (n) *n = h->f.n;
    if (p) *p = h->f.p;
    if (kind) *kind = h->f.kind;
    if (q) *q = h->f.q;
    if (log2m) *log2m = h->f.log2m;
    return RQ_OK;
}

int rq_hadamard_dense(const rq_hadamard_t* h, int8_t* host_out) {
    if (!h || !host_out || h->f.n > 8192) return RQ_ERR_ARG;
    const int n = h->f.n, p = h->f.p, m = 1 << h->f.log2m;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            host_out[(size_t)i * n + j] = (int8_t)(h->block[(size_t)(i / m) * p + (j / m)] *
                                                   rq::sylvester_entry(i % m, j % m));
    return RQ_OK;
}

int rq_next_order(int d, int* n_out) {
    if (d < 1 || !n_out) return RQ_ERR_ARG;
    for (int64_t n = ((int64_t)d + 31) / 32 * 32; n <= (1 << 30); n += 32) {
        rq::Factorisation f;
        if (rq::factor_order((int)n, &f) && f.log2m >= 5 && f.p <= rq::kMaxPaleyOrder) {
            *n_out = (int)n;
            return RQ_OK;
        }
    }
    return RQ_ERR_NO_ORDER;
}

int rq_hadamard_set_variant(rq_hadamard_t* h, int variant) {
    if (!h || variant < 0 || variant > 4) return RQ_ERR_ARG;
    h->variant = variant == 1 ? 1 : 0;
    h->split = variant == 2 ? -1 : variant == 3 ? 2 : variant == 4 ? 4 : 0;
    return RQ_OK;
}

const char* rq_hadamard_last_kernel(const rq_hadamard_t* h) {
    return h ? h->last_kernel.load(std::memory_order_relaxed) : "";
}

int rq_rotate_quantize(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d,
                       int64_t ld, int bits, float clip, void* codes, float* scales, void* stream) {
    int rc = check_rows(h, X, dtype, rows, d, ld, bits);
    if (rc != RQ_OK) return rc;
    if (!clip_ok(clip)) return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!codes || !scales || !aligned(codes, 4) || !aligned(scales, 4)) return RQ_ERR_ARG;
    if (h->device < 0) return RQ_ERR_HIP;
    const rq::RowArgs a = row_args(h, X, dtype, rows, d, ld, bits);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (h->variant == 0 && rq::wave_supports(h, a)) {
        note(h, "wave_sylvester");
        return rq::wave_rotate_quantize(h, a, clip, static_cast<uint32_t*>(codes), scales, s);
    }
    if (h->variant == 0 && rq::wave_block_supports(h, a)) {
        note(h, "wave_block");
        return rq::wave_block_rotate_quantize(h, a, clip, static_cast<uint32_t*>(codes), scales, s);
    }
    if (h->variant == 0 && rq::wave_block2_supports(h, a)) {
        note(h, "wave_block");
        return rq::wave_block2_rotate_quantize(h, a, clip, static_cast<uint32_t*>(codes), scales, s);
    }
    if (h->variant == 0 && rq::wg_block_supports(h, a)) {
        note(h, "wg_block");
        return rq::wg_block_rotate_quantize(h, a, clip, static_cast<uint32_t*>(codes), scales, s);
    }
    if (h->variant == 0 && rq::dense_block_supports(h, a)) {
        note(h, "dense_block");
        return rq::dense_block_rotate_quantize(h, a, clip, static_cast<uint32_t*>(codes), scales, s);
    }
    if (!rq::generic_supports(h)) return RQ_ERR_NO_ORDER;
    note(h, "generic_lds");
    return rq::generic_rotate_quantize(h, a, clip, static_cast<uint32_t*>(codes), scales, s);
}

int rq_rotate_quantize_asym(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d,
                            int64_t ld, int bits, float clip, void* codes, float* scales,
                            float* mins, void* stream) {
    int rc = check_rows(h, X, dtype, rows, d, ld, bits);
    if (rc != RQ_OK) return rc;
    if (!clip_ok(clip) || h->f.n % RQ_GROUP != 0) return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!codes || !scales || !mins || !aligned(codes, 4) || !aligned(scales, 4) || !aligned(mins, 4))
        return RQ_ERR_ARG;
    if (h->device < 0) return RQ_ERR_HIP;
    const rq::RowArgs a = row_args(h, X, dtype, rows, d, ld, bits);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (h->variant == 0 && rq::wave_asym_supports(h, a)) {
        note(h, "wave_short_asym");
        return rq::wave_rotate_quantize_asym(h, a, clip, static_cast<uint32_t*>(codes), scales, mins, s);
    }
    if (!rq::generic_supports(h)) return RQ_ERR_NO_ORDER;
    note(h, "generic_lds_asym");
    return rq::generic_rotate_quantize_asym(h, a, clip, static_cast<uint32_t*>(codes), scales, mins, s);
}

int rq_stream_reference(const void* X, int64_t rows, int n, int64_t ld, int bits, void* codes,
                        float* scales, void* stream) {
    if (rows < 0 || n < 512 || n > 8192 || n % 512 != 0 || ld < n || ld % 8 != 0 || (bits != 3 && bits != 4))
        return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!X || !codes || !scales || !aligned(X, 16) || !aligned(codes, 4) || !aligned(scales, 4)) return RQ_ERR_ARG;
    return rq::stream_reference(X, rows, n, ld, bits, static_cast<uint32_t*>(codes), scales,
                                static_cast<hipStream_t>(stream));
}

int rq_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                void* codes, float* scales, void* stream) {
    if (dtype != RQ_BF16 && dtype != RQ_F32 && dtype != RQ_F16) return RQ_ERR_ARG;
    if (rows < 0 || d < 32 || d % 32 != 0 || ld < d) return RQ_ERR_ARG;
    if (bits != 3 && bits != 4) return RQ_ERR_ARG;
    if (!clip_ok(clip)) return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!X || !aligned(X, dtype == RQ_F32 ? 4 : 2)) return RQ_ERR_ARG;
    if (!codes || !scales || !aligned(codes, 4) || !aligned(scales, 4)) return RQ_ERR_ARG;
    if (rq::plain_wave_short_supports(X, dtype, d, ld))     // head rows of 128 / 256 / 512: the short-row passes
        return rq::plain_wave_short_quantize(X, dtype, rows, d, ld, bits, clip, static_cast<uint32_t*>(codes), scales,
                                             static_cast<hipStream_t>(stream));
    if (rq::plain_short_supports(X, dtype, d, ld))          // other short rows: several rows per wave
        return rq::plain_short_quantize(X, dtype, rows, d, ld, bits, clip, static_cast<uint32_t*>(codes), scales,
                                        static_cast<hipStream_t>(stream));
    if (rq::plain_wave_supports(X, dtype, d, ld))
        return rq::plain_wave_quantize(X, dtype, rows, d, ld, bits, clip, static_cast<uint32_t*>(codes), scales,
                                       static_cast<hipStream_t>(stream));
    return rq::plain_quantize(X, dtype, rows, d, ld, bits, clip, static_cast<uint32_t*>(codes), scales,
                              static_cast<hipStream_t>(stream));
}

int rq_quantize_asym(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                     void* codes, float* scales, float* mins, void* stream) {
    if (dtype != RQ_BF16 && dtype != RQ_F32 && dtype != RQ_F16) return RQ_ERR_ARG;
    if (rows < 0 || d < RQ_GROUP || d % RQ_GROUP != 0 || ld < d) return RQ_ERR_ARG;
    if (bits != 3 && bits != 4) return RQ_ERR_ARG;
    if (!clip_ok(clip)) return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!X || !aligned(X, dtype == RQ_F32 ? 4 : 2)) return RQ_ERR_ARG;
    if (!codes || !scales || !mins || !aligned(codes, 4) || !aligned(scales, 4) || !aligned(mins, 4)) return RQ_ERR_ARG;
    return rq::plain_quantize_asym(X, dtype, rows, d, ld, bits, clip, static_cast<uint32_t*>(codes), scales, mins,
                                   static_cast<hipStream_t>(stream));
}

int rq_rotate(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
              int transpose, void* Y, int out_dtype, int d_out, int64_t ld_out, void* stream) {
    int rc = check_rows(h, X, dtype, rows, d, ld, 4);
    if (rc != RQ_OK) return rc;
    if (out_dtype != RQ_BF16 && out_dtype != RQ_F32 && out_dtype != RQ_F16) return RQ_ERR_ARG;
    if (d_out < 1 || d_out > h->f.n || ld_out < d_out || (transpose != 0 && transpose != 1))
        return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!Y || !aligned(Y, out_dtype == RQ_F32 ? 4 : 2)) return RQ_ERR_ARG;
    if (h->device < 0) return RQ_ERR_HIP;
    const rq::RowArgs a = row_args(h, X, dtype, rows, d, ld, 4);
    const rq::OutArgs o{Y, out_dtype, d_out, ld_out};
    if (h->variant == 0 && rq::wave_rotate_supports(h, a, o)) {      // Sylvester orders: H is symmetric
        note(h, "wave_rotate");
        return rq::wave_rotate(h, a, o, static_cast<hipStream_t>(stream));
    }
    if (h->variant == 0 && rq::wave_block_rotate_supports(h, a, transpose, o)) {
        note(h, "wave_block_rotate");
        return rq::wave_block_rotate(h, a, transpose, o, static_cast<hipStream_t>(stream));
    }
    if (!rq::generic_supports(h)) return RQ_ERR_NO_ORDER;
    note(h, "generic_rotate");
    return rq::generic_rotate(h, a, transpose, o, static_cast<hipStream_t>(stream));
}

int rq_dequantize_rotate(const rq_hadamard_t* h, const void* codes, const float* scales,
                         const float* mins, int64_t rows, int bits, int transpose, void* Y,
                         int out_dtype, int d_out, int64_t ld_out, void* stream) {
    if (!h || rows < 0 || (bits != 3 && bits != 4)) return RQ_ERR_ARG;
    if (out_dtype != RQ_BF16 && out_dtype != RQ_F32 && out_dtype != RQ_F16) return RQ_ERR_ARG;
    if (d_out < 1 || d_out > h->f.n || ld_out < d_out || (transpose != 0 && transpose != 1))
        return RQ_ERR_ARG;
    if (mins && h->f.n % RQ_GROUP != 0) return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!codes || !scales || !Y || !aligned(codes, 4) || !aligned(scales, 4) || !aligned(mins, 4) ||
        !aligned(Y, out_dtype == RQ_F32 ? 4 : 2))
        return RQ_ERR_ARG;
    if (h->device < 0) return RQ_ERR_HIP;
    const rq::RowArgs a = row_args(h, nullptr, RQ_F32, rows, h->f.n, h->f.n, bits);
    const rq::OutArgs o{Y, out_dtype, d_out, ld_out};
    if (h->variant == 0 && rq::wave_dequant_rotate_supports(h, a, mins, o)) {   // Sylvester orders: H is symmetric
        note(h, "wave_dequant_rotate");
        return rq::wave_dequant_rotate(h, a, static_cast<const uint32_t*>(codes), scales, mins, o,
                                       static_cast<hipStream_t>(stream));
    }
    if (!rq::generic_supports(h)) return RQ_ERR_NO_ORDER;
    note(h, "generic_dequant_rotate");
    return rq::generic_dequant_rotate(h, a, static_cast<const uint32_t*>(codes), scales, mins, transpose,
                                      o, static_cast<hipStream_t>(stream));
}

static int dequantize_impl(const rq_hadamard_t* h, const void* codes, const float* scales, const float* mins,
                           bool asym, int64_t rows, int bits, float* Y, void* stream) {
    if (!h || rows < 0 || (bits != 3 && bits != 4)) return RQ_ERR_ARG;
    if (asym && h->f.n % RQ_GROUP != 0) return RQ_ERR_ARG;
    if (rows == 0) return RQ_OK;
    if (!codes || !scales || !Y || (asym && !mins)) return RQ_ERR_ARG;
    if (!aligned(codes, 4) || !aligned(scales, 4) || !aligned(mins, 4) || !aligned(Y, 4)) return RQ_ERR_ARG;
    if (h->device < 0) return RQ_ERR_HIP;
    note(h, "dequantize");
    return rq::dequantize_rows(static_cast<const uint32_t*>(codes), scales, asym ? mins : nullptr, rows, h->f.n,
                               bits, Y, static_cast<hipStream_t>(stream));
}

int rq_dequantize(const rq_hadamard_t* h, const void* codes, const float* scales, int64_t rows, int bits,
                  float* Y, void* stream) {
    return dequantize_impl(h, codes, scales, nullptr, false, rows, bits, Y, stream);
}

int rq_dequantize_asym(const rq_hadamard_t* h, const void* codes, const float* scales, const float* mins,
                       int64_t rows, int bits, float* Y, void* stream) {
    return dequantize_impl(h, codes, scales, mins, true, rows, bits, Y, stream);
}

int rq_expand_limit(int n, int bits, int bits_reduced, int64_t* d_max) {
    if (!d_max || n < 1 || bits_reduced < 1 || bits_reduced > bits || bits > 64) return RQ_ERR_ARG;
    *d_max = ((int64_t)n * (bits - bits_reduced)) / bits_reduced;
    return RQ_OK;
}

size_t rq_quant_error_workspace(int64_t rows, int n_clips) {
    if (rows < 0 || n_clips < 1 || n_clips > RQ_MAX_CLIPS) return 0;
    size_t r = rows > 0 ? (size_t)rows : 1;
    return r * (size_t)n_clips * sizeof(double);
}

}  // extern "C"

int rq::quant_error_impl(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d,
                         int64_t ld, int bits, const float* clips, int n_clips, float* mse,
                         void* workspace, size_t workspace_bytes, void* stream, bool asym) {
    int rc = check_rows(h, X, dtype, rows, d, ld, bits);
    if (rc != RQ_OK) return rc;
    if (asym && h->f.n % RQ_GROUP != 0) return RQ_ERR_ARG;
    if (!clips || n_clips < 1 || n_clips > RQ_MAX_CLIPS) return RQ_ERR_ARG;
    if (!mse || !aligned(mse, 4) || !workspace || !aligned(workspace, 8)) return RQ_ERR_ARG;
    if (workspace_bytes < rq_quant_error_workspace(rows, n_clips)) return RQ_ERR_ARG;
    rq::ClipList cl;
    std::memset(&cl, 0, sizeof cl);
    for (int k = 0; k < n_clips; ++k) {
        if (!clip_ok(clips[k])) return RQ_ERR_ARG;
        cl.v[k] = clips[k];
        const double lvl = (double)((1 << bits) - 1);
        cl.lvl_over_clip[k] = lvl / (double)clips[k];
        cl.clip_over_lvl[k] = (double)clips[k] / lvl;
    }
    if (h->device < 0) return RQ_ERR_HIP;
    const rq::RowArgs a = row_args(h, X, dtype, rows, d, ld, bits);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (asym) {
        if (h->variant == 0 && rows > 0 && rq::wave_asym_supports(h, a)) {
            note(h, "wave_quant_error_asym");
            rc = rq::wave_quant_error_asym(h, a, cl, n_clips, static_cast<double*>(workspace), s);
            if (rc != RQ_OK) return rc;
            return rq::reduce_partials(static_cast<double*>(workspace), rows, n_clips, mse, s);
        }
        if (!rq::generic_supports(h)) return RQ_ERR_NO_ORDER;
        note(h, "generic_lds_asym");
        return rq::generic_quant_error_asym(h, a, cl, n_clips, mse, static_cast<double*>(workspace), s);
    }
    if (h->variant == 0 && rows > 0 && rq::wave_quant_error_supports(h, a)) {
        note(h, "wave_quant_error");
        rc = rq::wave_quant_error(h, a, cl, n_clips, static_cast<double*>(workspace), s);
        if (rc != RQ_OK) return rc;
        return rq::reduce_partials(static_cast<double*>(workspace), rows, n_clips, mse, s);
    }
    if (h->variant == 0 && rows > 0 && rq::wg_block_supports(h, a, true)) {
        note(h, "wg_block_quant_error");
        rc = rq::wg_block_quant_error(h, a, cl, n_clips, static_cast<double*>(workspace), s);
        if (rc != RQ_OK) return rc;
        return rq::reduce_partials(static_cast<double*>(workspace), rows, n_clips, mse, s);
    }
    if (!rq::generic_supports(h)) return RQ_ERR_NO_ORDER;
    note(h, "generic_lds");
    return rq::generic_quant_error(h, a, cl, n_clips, mse, static_cast<double*>(workspace), s);
}

extern "C" {

int rq_quant_error(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d,
                   int64_t ld, int bits, const float* clips, int n_clips, float* mse,
                   void* workspace, size_t workspace_bytes, void* stream) {
    return rq::quant_error_impl(h, X, dtype, rows, d, ld, bits, clips, n_clips, mse, workspace, workspace_bytes,
                            stream, false);
}

int rq_quant_error_asym(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d,
                        int64_t ld, int bits, const float* clips, int n_clips, float* mse,
                        void* workspace, size_t workspace_bytes, void* stream) {
    return rq::quant_error_impl(h, X, dtype, rows, d, ld, bits, clips, n_clips, mse, workspace, workspace_bytes,
                                stream, true);
}

namespace {
// Probes evaluated per batch of the search: 5 steps ahead (the 31 nodes of the outcome tree, plus the
// starting point in the first batch) on small tensors, 3 steps (7 nodes + 1) on large ones, where the
// extra candidates would cost more than the launches they save.
constexpr int64_t kGbsSmall = (int64_t)1 << 22;              // rows * n up to which 5 steps are taken
int gbs_depth(int64_t rows, int n) { return (double)rows * (double)n <= (double)kGbsSmall ? 5 : 3; }
}  // namespace

size_t rq_gbs_workspace(int64_t rows) {
    if (rows < 0) return 0;
    // the order is not known here: with the smallest one (32) more than 2^22 / 32 rows always take 3 steps
    const int cands = rows * 32 <= kGbsSmall ? 32 : 8;
    const size_t q = rq_quant_error_workspace(rows, cands);
    return q ? q + 256 : 0;
}

namespace {

// State of Algorithm 1's inner loop (section 4.1): bracket [a, b], best point m, iteration parity.
// RQ_MAX_CLIPS floats of pinned host memory and their device address, one buffer per host thread and device,
// allocated at the first search of that thread on that device and kept until the process ends (a search is a
// host loop that synchronises its stream, so the buffer is never in use by two searches at once).
struct MappedVals {
    float* host = nullptr;
    float* dev = nullptr;
};

MappedVals mapped_vals(int device) {
    struct Entry { int device; MappedVals mv; };
    thread_local std::vector<Entry> cache;
    for (const Entry& e : cache)
        if (e.device == device) return e.mv;
    MappedVals mv;
    int cur = -1;
    void* hp = nullptr;
    void* dp = nullptr;
    if (hipGetDevice(&cur) == hipSuccess && cur == device &&
        hipHostMalloc(&hp, sizeof(float) * RQ_MAX_CLIPS, hipHostMallocMapped) == hipSuccess) {
        if (hipHostGetDevicePointer(&dp, hp, 0) == hipSuccess && dp) {
            mv.host = static_cast<float*>(hp);
            mv.dev = static_cast<float*>(dp);
        } else {
            (void)hipHostFree(hp);
        }
    }
    (void)hipGetLastError();
    cache.push_back(Entry{device, mv});
    return mv;
}

// State of the search of Algorithm 1 (section 4.1): the best point so far and the nearest evaluated
// point on either side of it; probes go to the midpoint towards the left and the right neighbour in turn.
struct GbsState {
    double near[2];       // nearest evaluated points: [0] left of best, [1] right of best
    double best;
    int side;             // neighbour the next probe goes towards
    double width() const { return near[1] - near[0]; }
    double probe() const { return 0.5 * (near[side] + best); }
    // after probing x = probe(): `better` = the probe beat the best point, which then bounds the far side
    GbsState next(double x, bool better) const {
        GbsState n = *this;
        if (better) {
            n.near[1 - side] = best;
            n.best = x;
        } else {
            n.near[side] = x;
        }
        n.side = 1 - side;
        return n;
    }
};

// Probes of the next `depth` steps for every outcome of the comparisons on the way, in heap order
// (node i: children 2 i for "better", 2 i + 1 for "not better"); the positions do not depend on the
// objective values, only on the outcomes.  x[i] < 0 marks a node the search cannot reach.
void gbs_tree(const GbsState& st, double eps, int depth, int idx, double* x) {
    if (depth == 0 || st.width() <= eps) return;
    const double p = st.probe();
    x[idx] = p;
    gbs_tree(st.next(p, true), eps, depth - 1, 2 * idx, x);
    gbs_tree(st.next(p, false), eps, depth - 1, 2 * idx + 1, x);
}

}  // namespace

static int gbs_impl(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
                    int bits, float eps, int max_evals, void* workspace, size_t workspace_bytes,
                    void* stream, float* clip_out, float* mse_out, float* trace_clips,
                    float* trace_mse, int* n_evals, bool asym) {
    int rc = check_rows(h, X, dtype, rows, d, ld, bits);
    if (rc != RQ_OK) return rc;
    if (asym && h->f.n % RQ_GROUP != 0) return RQ_ERR_ARG;
    if (rows < 1 || !(eps > 0.0f) || max_evals < 1 || max_evals > 256) return RQ_ERR_ARG;
    if (!clip_out || !mse_out || !workspace || !aligned(workspace, 8)) return RQ_ERR_ARG;
    if (workspace_bytes < rq_gbs_workspace(rows)) return RQ_ERR_ARG;
    if (h->device < 0) return RQ_ERR_HIP;
    // layout of the workspace: [0, 256) the objective values of one batch, then the quant_error scratch
    float* d_mse = static_cast<float*>(workspace);
    void* qws = static_cast<char*>(workspace) + 256;
    const size_t qws_bytes = workspace_bytes - 256;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // The probes of Algorithm 1 are taken in the listing's order, but evaluated ahead of time in
    // batches: one quant_error launch covers every probe the next `depth` steps can ask for (a binary
    // tree over the comparison outcomes), then the host walks the tree with the values.  The values
    // and the sequence of probes are those of the one-at-a-time loop; what changes is the number of
    // launches and stream synchronisations (each costs more than a candidate on a small tensor).
    // Small tensors look 5 steps ahead (31 candidates), large ones 3 (7 candidates: about the work
    // of the 3 rotations it saves).
    const int depth = gbs_depth(rows, h->f.n);
    float vals[RQ_MAX_CLIPS];
    float clips[RQ_MAX_CLIPS];
    // The objective values of a batch come back through pinned host memory that the reduction kernel writes
    // itself (mapped into the device's address space): a batch then costs one synchronisation of the caller's
    // stream and no copy.  Where that memory cannot be had, they are copied back on the same stream.
    const MappedVals mv = mapped_vals(h->device);
    auto evaluate = [&](int count) -> int {
        float* out = mv.dev ? mv.dev : d_mse;
        int r = rq::quant_error_impl(h, X, dtype, rows, d, ld, bits, clips, count, out, qws, qws_bytes, stream, asym);
        if (r != RQ_OK) return r;
        if (mv.dev) {
            if (hipStreamSynchronize(s) != hipSuccess) return RQ_ERR_HIP;
            std::memcpy(vals, mv.host, sizeof(float) * count);
            return RQ_OK;
        }
        // read back on the caller's stream: no other stream is made to wait
        if (hipMemcpyAsync(vals, d_mse, sizeof(float) * count, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return RQ_ERR_HIP;
        return RQ_OK;
    };
    int evals = 0;
    auto record = [&](float c, float v) {
        if (trace_clips) trace_clips[evals] = c;
        if (trace_mse) trace_mse[evals] = v;
        ++evals;
    };
    GbsState st{{0.0, 1.0}, 0.5, 0};
    float fm = 0.0f;
    bool first = true;
    while (first || (st.width() > (double)eps && evals < max_evals)) {
        double x[64];
        int slot[64];
        for (int i = 0; i < 64; ++i) x[i] = -1.0;
        gbs_tree(st, (double)eps, depth, 1, x);
        int count = 0;
        if (first) clips[count++] = (float)st.best;          // the starting point rides along with the first batch
        for (int i = 1; i < (1 << depth); ++i)
            if (x[i] >= 0.0) {
                slot[i] = count;
                clips[count++] = (float)x[i];
            }
        if (count == 0) break;
        rc = evaluate(count);
        if (rc != RQ_OK) return rc;
        if (first) {
            fm = vals[0];
            record(clips[0], fm);
            first = false;
        }
        int idx = 1;
        for (int lvl = 0; lvl < depth && st.width() > (double)eps && evals < max_evals; ++lvl) {
            const double p = x[idx];
            const float fx = vals[slot[idx]];
            record((float)p, fx);
            const bool better = fx < fm;
            if (better) fm = fx;
            st = st.next(p, better);
            idx = 2 * idx + (better ? 0 : 1);
        }
    }
    *clip_out = (float)st.best;
    *mse_out = fm;
    if (n_evals) *n_evals = evals;
    return RQ_OK;
}

int rq_gbs_search(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
                  int bits, float eps, int max_evals, void* workspace, size_t workspace_bytes,
                  void* stream, float* clip_out, float* mse_out, float* trace_clips,
                  float* trace_mse, int* n_evals) {
    return gbs_impl(h, X, dtype, rows, d, ld, bits, eps, max_evals, workspace, workspace_bytes, stream,
                    clip_out, mse_out, trace_clips, trace_mse, n_evals, false);
}

int rq_gbs_search_asym(const rq_hadamard_t* h, const void* X, int dtype, int64_t rows, int d, int64_t ld,
                       int bits, float eps, int max_evals, void* workspace, size_t workspace_bytes,
                       void* stream, float* clip_out, float* mse_out, float* trace_clips,
                       float* trace_mse, int* n_evals) {
    return gbs_impl(h, X, dtype, rows, d, ld, bits, eps, max_evals, workspace, workspace_bytes, stream,
                    clip_out, mse_out, trace_clips, trace_mse, n_evals, true);
}

const char* rq_strerror(int code) {
    switch (code) {
        case RQ_OK: return "ok";
        case RQ_ERR_ARG: return "invalid argument";
        case RQ_ERR_NO_ORDER: return "no supported Hadamard order";
        case RQ_ERR_HIP: return "HIP failure or handle without device tables";
        case RQ_ERR_NOMEM: return "out of host memory";
        case RQ_ERR_TOO_LARGE: return "input larger than the static scratch buffer of the no-allocation call";
        default: return "unknown error";
    }
}

}  // extern "C"
