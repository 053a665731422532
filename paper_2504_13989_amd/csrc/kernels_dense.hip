// Dense-block kernel: bf16 rows of an order n <= 4096 whose factorisation leaves no long
// power-of-two axis for the wave kernels - above all a large Paley block taken over the whole
// dimension (1544 = 1543 + 1, the 1536 + 8 expansion of section 5.2.2), also p * 2^k with k < 7.
// Here the rotation really is a dense contraction, y = H_n x with n multiply-adds per output
// (sections 2.3.3, 4.2), so it runs on the matrix cores as a GEMM: D[a'][row] = sum_a H[a'][a]
// X[row][a], v_mfma_f32_16x16x32_bf16 with
//   B operand  16 rows x 32 inputs as they are in memory: lane (g, r) takes the 16 bytes
//              X[row0 + r][32 kk + 8 g ..] (exact bf16, no conversion), staged through LDS so that the
//              loads from memory are coalesced (see the loader role in the kernel);
//   A operand  a 16 x 32 tile of +-1 (bf16), made in registers from one sign bit per entry: the handle
//              holds the matrix as n^2 / 8 bytes of signs, a lane's 8 signs of a tile sit in a 32-bit word
//              (four tiles per word) at the positions where one rotation of the word brings two of them
//              to bits 15 and 31, so an operand register costs a rotate and an and-or:
//              8 vector instructions per tile against 16 NT matrix-core cycles;
//   D          lane (g, r) register j = output 16 mt + 4 g + j of row r, fp32.
// A workgroup of 8 waves owns 16 NT rows (NT = 1, or 2 when there are rows enough: every tile then serves
// two groups of rows); wave w owns the output tiles mt = w, w + 8, ... and keeps their accumulators in
// registers over the whole contraction.  Then: row absmax (registers, the four lane rows, the
// eight waves through LDS), scale, round/clamp (section 2.1 with the clip ratio of section 3.1),
// pack into an LDS image of the packed rows, copy out coalesced.
// A wave reads 16 bytes of signs per lane and contraction step (n^2 / 8 bytes per workgroup in all,
// against 2 n^2 when the table held bf16 tiles and the kernel was bound by reading them from the L2
// cache): what is left is the matrix cores and the vector instructions that feed them.
#include "wave_common.h"

namespace rq {
namespace {

constexpr int kDenseWaves = 8;

// 32-bit sign words per lane and (contraction step, wave): four tiles per word, whole 16-byte loads
constexpr int dense_words(int mtw) { return mtw <= 16 ? 4 : 8; }

// Operand register d (entries 2 d, 2 d + 1 of the lane's eight) of the tile in slot jj of a sign word:
// the rotation by 4 jj + d brings their signs to bits 15 and 31.  `mask` (0x80008000) and `one`
// (0x3F803F80) are passed in registers so that the and-or is one instruction.
template <int RHO>
__device__ __forceinline__ uint32_t sign_pair(uint32_t word, uint32_t mask, uint32_t one) {
    const uint32_t x = RHO ? __builtin_amdgcn_alignbit(word, word, RHO) : word;
    return (x & mask) | one;
}

template <int JJ>
__device__ __forceinline__ u32x4 sign_tile(uint32_t word, uint32_t mask, uint32_t one) {
    return u32x4{sign_pair<4 * JJ>(word, mask, one), sign_pair<4 * JJ + 1>(word, mask, one),
                 sign_pair<4 * JJ + 2>(word, mask, one), sign_pair<4 * JJ + 3>(word, mask, one)};
}

// Steps of the contraction per group: the rows' chunks of a group (64 kDenseGroup bytes per row) are staged
// in LDS at once, and the sign table is padded to whole groups plus one.
constexpr int kDenseGroup = 4;
constexpr int dense_steps_padded(int n) { return (((n + 31) / 32 + kDenseGroup - 1) / kDenseGroup + 1) * kDenseGroup; }

template <int MTW, int NT, int BITS>
__global__ __launch_bounds__(64 * kDenseWaves) void k_dense_block(WaveArgs a, int n) {
    constexpr int RB = 16 * NT;                          // rows per workgroup
    constexpr int QV = dense_words(MTW) / 4;             // 16-byte sign loads per lane and step
    constexpr int G = kDenseGroup;
    constexpr int CPR = 4 * G;                           // 16-byte chunks per row and group
    constexpr int PITCH = 64 * G + 16;                   // LDS bytes per staged row: 16 rows apart = 16 different banks
    // LDS: two staging buffers of RB rows x PITCH while the contraction runs, then the RB packed rows
    extern __shared__ __attribute__((aligned(16))) uint8_t stage[];
    __shared__ float wmax[kDenseWaves][RB];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, r = lane & 15;
    const int MT = (n + 15) >> 4, KK = (n + 31) >> 5;
    const int NG = (KK + G - 1) / G;
    const int row_bytes = n * BITS / 8;
    const int64_t row0 = (int64_t)blockIdx.x * RB;
    bool row_ok[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) row_ok[q] = row0 + 16 * q + r < a.rows;
    uint32_t kmask = 0x80008000u, kone = 0x3F803F80u;
    asm volatile("" : "+v"(kmask), "+v"(kone));          // kept in registers, see sign_pair
    const u32x4* const signs = a.tiles + ((size_t)wave * 64 + lane) * QV;     // + kk * 8 * 64 * QV

    // Loader role: thread t brings chunk t % CPR of row t / CPR of every group from memory - 16 consecutive
    // lanes read 256 consecutive bytes - and puts it into LDS, where lane (g, r) of every wave finds the
    // operand chunks of its rows.  (Loading the operands directly, lane (g, r) from row r, makes every lane
    // of a load instruction a different cache line: measured, the address path then takes longer than the
    // matrix cores.)  A chunk beyond the row's d inputs, or of a row beyond the last, is zero
    // (section 4.2): its load goes to an address inside X and the zero is put in on the way to LDS.
    const int lrow = threadIdx.x / CPR, lchunk = threadIdx.x % CPR;
    const bool loader = lrow < RB;
    const bool lrow_ok = loader && row0 + lrow < a.rows;
    const uint16_t* const lptr = a.X + (lrow_ok ? row0 + lrow : 0) * a.ld;
    uint8_t* const lds_w = stage + (loader ? lrow : 0) * PITCH + lchunk * 16;
    const uint8_t* const lds_r = stage + r * PITCH + g * 16;
    auto gload = [&](int grp) {
        const int e = (grp * CPR + lchunk) * 8;
        return *reinterpret_cast<const u32x4*>(lptr + (e < a.d ? e : 0));
    };
    auto lds_store = [&](int grp, u32x4 v) {
        const int e = (grp * CPR + lchunk) * 8;
        if (!(lrow_ok && e < a.d)) v = u32x4{0u, 0u, 0u, 0u};
        if (loader) *reinterpret_cast<u32x4*>(lds_w + (grp & 1) * (RB * PITCH)) = v;
    };

    f32x4 acc[MTW][NT];
#pragma unroll
    for (int j = 0; j < MTW; ++j)
#pragma unroll
        for (int q = 0; q < NT; ++q) acc[j][q] = f32x4{0.f, 0.f, 0.f, 0.f};

    // tile slots of a wave beyond the matrix (mt >= MT) are computed like the others - their signs read as
    // +1 - so that a step is one straight run of instructions; their outputs are never used.  Entries of a
    // tile beyond column n meet the zero chunks of X.
    auto contract = [&](const u32x4 (&sg)[QV], const u32x4 (&x)[NT]) {
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const uint32_t word = sg[j / 16][(j / 4) % 4];
            const u32x4 t = (j % 4) == 0   ? sign_tile<0>(word, kmask, kone)
                            : (j % 4) == 1 ? sign_tile<1>(word, kmask, kone)
                            : (j % 4) == 2 ? sign_tile<2>(word, kmask, kone)
                                           : sign_tile<3>(word, kmask, kone);
#pragma unroll
            for (int q = 0; q < NT; ++q)
                acc[j][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t),
                                                                    __builtin_bit_cast(bf16x8, x[q]), acc[j][q], 0, 0, 0);
        }
        // issue order: the 8 vector instructions that make tile j + 1 go between the matrix-core instructions
        // of tile j (into other registers than tile j's, which those are still reading)
        __builtin_amdgcn_sched_group_barrier(0x2, 8, 0);
#pragma unroll
        for (int j = 0; j < MTW; ++j)
#pragma unroll
            for (int q = 0; q < NT; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x8, 1, 0);
                if (j + 1 < MTW) __builtin_amdgcn_sched_group_barrier(0x2, 8 / NT, 0);
            }
    };

    // Group n of the contraction: its sign words were requested a group earlier (registers), its chunks
    // of X are in LDS buffer n & 1; while it runs, the signs of group n + 1 are requested, the chunks of
    // group n + 1 (requested a group earlier) go to the other LDS buffer and those of group n + 2 are
    // requested.  Everything beyond the last group is padding: sign words of zeros, chunks masked to zero.
    u32x4 sC[G][QV], sN[G][QV];
    u32x4 R = gload(0);
#pragma unroll
    for (int i = 0; i < G; ++i)
#pragma unroll
        for (int v = 0; v < QV; ++v) sC[i][v] = signs[(size_t)i * (kDenseWaves * 64 * QV) + v];
    lds_store(0, R);
    R = gload(1);
    __syncthreads();
    for (int grp = 0; grp + 1 < NG; ++grp) {
#pragma unroll
        for (int i = 0; i < G; ++i)
#pragma unroll
            for (int v = 0; v < QV; ++v)
                sN[i][v] = signs[(size_t)((grp + 1) * G + i) * (kDenseWaves * 64 * QV) + v];
        const uint8_t* const rd = lds_r + (grp & 1) * (RB * PITCH);
        u32x4 xa[NT], xb[NT];                            // operands of the even / odd steps of the group
#pragma unroll
        for (int q = 0; q < NT; ++q) xa[q] = *reinterpret_cast<const u32x4*>(rd + 16 * q * PITCH);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < G; i += 2) {
#pragma unroll
            for (int q = 0; q < NT; ++q) xb[q] = *reinterpret_cast<const u32x4*>(rd + 16 * q * PITCH + (i + 1) * 64);
            __builtin_amdgcn_sched_barrier(0);
            contract(sC[i], xa);
            __builtin_amdgcn_sched_barrier(0);
            if (i + 2 < G) {
#pragma unroll
                for (int q = 0; q < NT; ++q)
                    xa[q] = *reinterpret_cast<const u32x4*>(rd + 16 * q * PITCH + (i + 2) * 64);
            }
            __builtin_amdgcn_sched_barrier(0);
            contract(sC[i + 1], xb);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_store(grp + 1, R);
        R = gload(grp + 2);
#pragma unroll
        for (int i = 0; i < G; ++i)
#pragma unroll
            for (int v = 0; v < QV; ++v) sC[i][v] = sN[i][v];
        __syncthreads();
    }
    {
        // last group: only the steps that exist (KK need not be a multiple of G), nothing left to request
        const int rem = KK - (NG - 1) * G;
        const uint8_t* const rd = lds_r + ((NG - 1) & 1) * (RB * PITCH);
#pragma unroll
        for (int i = 0; i < G; ++i) {
            if (i < rem) {
                u32x4 x[NT];
#pragma unroll
                for (int q = 0; q < NT; ++q) x[q] = *reinterpret_cast<const u32x4*>(rd + 16 * q * PITCH + i * 64);
                contract(sC[i], x);
            }
        }
        __syncthreads();                                 // the staging buffers become the packed rows' image
    }

    // absmax of the lane's rows: this lane's registers, the four lane rows, the eight waves
    float m[NT];
#pragma unroll
    for (int q = 0; q < NT; ++q) {
        float v = 0.0f;
#pragma unroll
        for (int j = 0; j < MTW; ++j)
            if (16 * (wave + kDenseWaves * j) + 4 * g < n) v = absmax4(v, acc[j][q]);   // outputs of the matrix only
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
    const size_t rows_lds = (size_t)16 * NT * n * bits / 8, stage_lds = (size_t)2 * 16 * NT * (64 * kDenseGroup + 16);
    const size_t lds = rows_lds > stage_lds ? rows_lds : stage_lds;
    if (bits == 4)
        hipLaunchKernelGGL((k_dense_block<MTW, NT, 4>), dim3((unsigned)groups), dim3(64 * kDenseWaves), lds, s, a, n);
    else
        hipLaunchKernelGGL((k_dense_block<MTW, NT, 3>), dim3((unsigned)groups), dim3(64 * kDenseWaves), lds, s, a, n);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

}  // namespace

// Sign table of the whole n x n matrix `hm` (row-major +-1) for k_dense_block: [kk][wave][lane][word],
// dense_words(tiles per wave) 32-bit words.  Lane (gA, mm) of wave w finds in word j / 4 the signs of its
// tile j (outputs 16 (w + 8 j) + mm, inputs 32 kk + 8 gA + i, i = 0..7; set = -1): with rho = 4 (j % 4) +
// i / 2, entry i sits at bit (15 + rho) % 32 when i is even and (31 + rho) % 32 when it is odd - the
// places that a rotation of the word by rho brings to bits 15 and 31.  Entries outside the matrix are 0.
std::vector<uint32_t> dense_block_tiles(const std::vector<int8_t>& hm, int n) {
    const int MT = (n + 15) / 16, KK = (n + 31) / 32;
    const int mtw = (MT + kDenseWaves - 1) / kDenseWaves, words = dense_words(mtw);
    std::vector<uint32_t> t((size_t)dense_steps_padded(n) * kDenseWaves * 64 * words, 0u);   // zeros beyond step KK
    for (int kk = 0; kk < KK; ++kk)
        for (int w = 0; w < kDenseWaves; ++w)
            for (int lane = 0; lane < 64; ++lane) {
                const int gA = lane >> 4, mm = lane & 15;
                uint32_t* out = &t[(((size_t)kk * kDenseWaves + w) * 64 + lane) * words];
                for (int j = 0; j < mtw; ++j) {
                    const int ao = 16 * (w + kDenseWaves * j) + mm;
                    for (int i = 0; i < 8; ++i) {
                        const int ai = 32 * kk + 8 * gA + i;
                        if (ao >= n || ai >= n || hm[(size_t)ao * n + ai] > 0) continue;
                        const int rho = 4 * (j % 4) + i / 2;
                        out[j / 4] |= 1u << (((i & 1) ? 31 + rho : 15 + rho) % 32);
                    }
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
    // 32 rows per workgroup: every operand tile made in registers then serves two groups of rows; used when
    // that still leaves a workgroup for every CU and the accumulators fit the register budget (two waves
    // per SIMD; 64 rows need 208 accumulator registers per wave and spill)
    const bool two = a.rows >= (int64_t)32 * h->num_cu;
#define RQ_DENSE_CASE(M) \
    if (mtw <= M) return two ? launch_dense<M, 2>(w, a.n, a.bits, s) : launch_dense<M, 1>(w, a.n, a.bits, s)
    RQ_DENSE_CASE(4);
    RQ_DENSE_CASE(6);
    RQ_DENSE_CASE(8);
    RQ_DENSE_CASE(10);
    RQ_DENSE_CASE(13);
#undef RQ_DENSE_CASE
    if (mtw <= 16) return launch_dense<16, 1>(w, a.n, a.bits, s);
    if (mtw <= 20) return launch_dense<20, 1>(w, a.n, a.bits, s);
    if (mtw <= 24) return launch_dense<24, 1>(w, a.n, a.bits, s);
    if (mtw <= 28) return launch_dense<28, 1>(w, a.n, a.bits, s);
    if (mtw <= 32) return launch_dense<32, 1>(w, a.n, a.bits, s);
    return RQ_ERR_NO_ORDER;
}

}  // namespace rq
