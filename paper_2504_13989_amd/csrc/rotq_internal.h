// Internal declarations shared by the C ABI layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <vector>

#include "../../include/rotq.h"
#include "hadamard.h"

struct rq_hadamard {
    rq::Factorisation f;
    std::vector<int8_t> block;       // host copy of H_p, row-major p x p
    int device = -1;                 // device the tables live on; -1 = host-only handle
    int8_t* d_block = nullptr;       // device copy of `block`
    void* d_tiles = nullptr;         // device MFMA operand tiles of the block stage (bf16)
    void* d_tiles_f16 = nullptr;     // the same tiles encoded in fp16 (wave kernels only)
    void* d_tiles_t = nullptr;       // blocks up to 32: operand tiles of the transposed block (rq_rotate with
    void* d_tiles_t_f16 = nullptr;   // transpose = 1), bf16 and fp16
    void* d_tiles2 = nullptr;        // blocks of 33 .. 64: operand tiles of the one-wave kernel (d_tiles holds the
    void* d_tiles2_f16 = nullptr;    // workgroup kernel's), bf16 and fp16
    int max_lds = 0;                 // bytes of LDS one workgroup may use on `device`
    int num_cu = 0;
    bool wg_ok = false;              // the workgroup block kernel is usable for this order
    bool dense_ok = false;           // d_tiles holds the whole matrix for the dense-block kernel
    bool generic_ok = false;         // the general LDS kernel can hold a row of this order
    bool generic_f64_ok = false;     // ... and an fp64 copy of it (how fp32 rows are quantized)
    // test / measurement hook (rq_hadamard_set_variant); atomic so that a hot-path call on another
    // thread reads a whole value
    std::atomic<int> variant{0};     // 0 auto, 1 general LDS kernel
    std::atomic<int> split{0};       // long Sylvester rows: 0 auto, 2 / 4 waves per row, -1 never split
    // diagnostic only: name of the kernel family the most recent hot-path call chose.  The hot-path
    // calls take the handle as const and may run on several host threads at once, hence atomic.
    mutable std::atomic<const char*> last_kernel{""};
};

namespace rq {

struct RowArgs {
    const void* X;
    int dtype;
    int64_t rows;
    int d;
    int64_t ld;
    int n, p, log2m;
    const int8_t* block;
    int bits;
};

struct OutArgs {
    void* Y;          // rows x d_out results, fp32 or bf16
    int dtype;
    int d_out;
    int64_t ld_out;
};

struct ClipList {
    float v[RQ_MAX_CLIPS];
    // row-independent factors of the candidate scales, formed once on the host in fp64:
    // levels / clip and clip / levels, levels = 2^b - 1
    double lvl_over_clip[RQ_MAX_CLIPS];
    double clip_over_lvl[RQ_MAX_CLIPS];
};

// General LDS kernels: one workgroup per row, any supported order that fits in LDS.
// Return RQ_OK / RQ_ERR_*.
int generic_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                            float* scales, hipStream_t s);
int generic_quant_error(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                        float* mse, double* partial, hipStream_t s);
int generic_rotate_quantize_asym(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                                 float* scales, float* mins, hipStream_t s);
// Rotation with a floating-point result (H_n or H_n^T), from rows or from packed codes.
int generic_rotate(const rq_hadamard* h, const RowArgs& a, int transpose, const OutArgs& o,
                   hipStream_t s);
int generic_dequant_rotate(const rq_hadamard* h, const RowArgs& a, const uint32_t* codes,
                           const float* scales, const float* mins, int transpose, const OutArgs& o,
                           hipStream_t s);
// Rotation-free per-token quantizer (any d that is a multiple of 32).
int plain_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                   uint32_t* codes, float* scales, hipStream_t s);
// The same on the wave path: bf16 rows up to 20480 wide, 16-byte aligned.
bool plain_wave_supports(const void* X, int dtype, int d, int64_t ld);
int plain_wave_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                        uint32_t* codes, float* scales, hipStream_t s);
// The same on head rows of 128 / 256 / 512 16-bit values: the short-row passes of the rotating kernels with the
// identity on the matrix cores.
bool plain_wave_short_supports(const void* X, int dtype, int d, int64_t ld);
int plain_wave_short_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                              uint32_t* codes, float* scales, hipStream_t s);
bool generic_supports(const rq_hadamard* h);
bool generic_prepare(rq_hadamard* h);

// Wave-per-row kernels (bf16 rows, Sylvester orders 128 .. 8192, 16-byte aligned rows).
std::vector<uint32_t> wave_sylvester_tiles();
// The +-1 entries of a bf16 operand table re-encoded as IEEE fp16.
std::vector<uint32_t> tiles_to_f16(const std::vector<uint32_t>& bf16_tiles);
bool wave_supports(const rq_hadamard* h, const RowArgs& a);
int wave_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                         float* scales, hipStream_t s);
// Asymmetric group-128 variant on the wave path: bf16 rows of order 128 (one group per row).
bool wave_asym_supports(const rq_hadamard* h, const RowArgs& a);
int wave_rotate_quantize_asym(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                              float* scales, float* mins, hipStream_t s);
// quant_error on the wave path (bf16, Sylvester orders 1024 .. 8192): fills partial[rows][n_clips];
// reduce_partials then averages over rows.
bool wave_quant_error_supports(const rq_hadamard* h, const RowArgs& a);
int wave_quant_error(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                     double* partial, hipStream_t s);
int wave_quant_error_asym(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                          double* partial, hipStream_t s);
int generic_quant_error_asym(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                             float* mse, double* partial, hipStream_t s);
int reduce_partials(double* partial, int64_t rows, int n_clips, float* mse, hipStream_t s);
// Block kernel: bf16 rows, n = pb * 128 with a +-1 block of order pb <= 32 (Paley (x) small
// Sylvester) on the matrix cores.
std::vector<uint32_t> wave_block_tiles(const std::vector<int8_t>& bm, int pb);
bool wave_block_supports(const rq_hadamard* h, const RowArgs& a);
int wave_block_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                               float* scales, hipStream_t s);

// Rotation alone for those orders (H_n, or H_n^T with the transposed block's tiles).
bool wave_block_rotate_supports(const rq_hadamard* h, const RowArgs& a, int transpose, const OutArgs& o);
int wave_block_rotate(const rq_hadamard* h, const RowArgs& a, int transpose, const OutArgs& o, hipStream_t s);

// One-wave block kernel for blocks of 33 .. 64 (n <= 8192): bf16 / fp16 rows, 16-byte aligned.
std::vector<uint32_t> wave_block2_tiles(const std::vector<int8_t>& bm, int pb);
bool wave_block2_supports(const rq_hadamard* h, const RowArgs& a);
int wave_block2_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                                float* scales, hipStream_t s);

// Rotation-free asymmetric group-128 quantizer: any input type; 16-byte loads when the rows allow.
bool plain_short_supports(const void* X, int dtype, int d, int64_t ld);
int plain_short_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                         uint32_t* codes, float* scales, hipStream_t s);
int plain_quantize_asym(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                        uint32_t* codes, float* scales, float* mins, hipStream_t s);

// Rotation alone on the wave path: 16-bit rows of Sylvester order 128 .. 8192, 16-byte aligned rows in and out.
bool wave_rotate_supports(const rq_hadamard* h, const RowArgs& a, const OutArgs& o);
int wave_rotate(const rq_hadamard* h, const RowArgs& a, const OutArgs& o, hipStream_t s);
// Packed codes (+ scales, + mins when a row is one group of 128) to rows in the original basis on the
// wave path: Sylvester orders 128 .. 8192.
bool wave_dequant_rotate_supports(const rq_hadamard* h, const RowArgs& a, const float* mins, const OutArgs& o);
int wave_dequant_rotate(const rq_hadamard* h, const RowArgs& a, const uint32_t* codes, const float* scales,
                        const float* mins, const OutArgs& o, hipStream_t s);

// Dense-block kernel: bf16 rows, any order n <= 4096 that the wave kernels do not serve (the whole
// matrix on the matrix cores), e.g. 1544 as one Paley block.
std::vector<uint32_t> dense_block_tiles(const std::vector<int8_t>& hm, int n);
bool dense_block_supports(const rq_hadamard* h, const RowArgs& a);
int dense_block_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                                float* scales, hipStream_t s);

// Workgroup block kernel: bf16 or fp16 rows, n = pb * 128 with 32 < pb <= 256 (e.g. 18944 = 148 * 128),
// or n = p * 64 / p * 32 with 4 <= p <= 256 (several rows per pass); quant_error: the former, bf16.
std::vector<uint32_t> wg_block_tiles(const std::vector<int8_t>& bm, int pb);
bool wg_block_prepare(int pb);
bool wg_block_supports(const rq_hadamard* h, const RowArgs& a, bool quant_error = false);
int wg_block_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                             float* scales, hipStream_t s);
int wg_block_quant_error(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                         double* partial, hipStream_t s);

// The shared body of rq_quant_error / rq_quant_error_asym (argument checks, dispatch, reduction).
int quant_error_impl(const rq_hadamard* h, const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits,
                     const float* clips, int n_clips, float* mse, void* workspace, size_t workspace_bytes,
                     void* stream, bool asym);

// Device address of the library's static scratch array on device `dev`; the first call for a device must
// be made with that device current (rq_hadamard_build does so).  nullptr when it cannot be resolved.
void* static_scratch(int dev);

// Codes (+ scales, + mins) to values in the rotated domain, no rotation.
int dequantize_rows(const uint32_t* codes, const float* scales, const float* mins, int64_t rows, int n, int bits,
                    float* Y, hipStream_t s);

// Traffic-only reference kernel (measurement aid): rows of n = 512 T 16-bit values.
int stream_reference(const void* X, int64_t rows, int n, int64_t ld, int bits, uint32_t* codes, float* scales,
                     hipStream_t s);

}  // namespace rq
