// Workgroup block kernel: bf16 rows of order n = pb * 128 with a +-1 block of order
// 32 < pb <= 256 along the strided axis (H_n = B (x) H_128, B = H_p (x) H_{2^(k-7)}; sections
// 2.3.2, 2.3.3) - e.g. 18944 = 148 * 128 with the order-148 Paley II block; also the Sylvester
// orders 2^14 and 2^15, which are too long for one wave (B = H_128, H_256).
//
// The dense block product Y1[pb x 128] = B * X[pb x 128] is a real contraction (pb adds per
// output), so it runs on the matrix cores.  NW = ceil(pb / 16) waves share a row, wave w owning
// the 16 block rows 16 w .. 16 w + 15 on input and on output:
//   phase 1  the wave loads its block rows (16-byte chunks, 4 per lane), transposes 16-bit
//            values inside each lane (v_perm_b32) so that consecutive block rows of one column are
//            adjacent, and writes them to LDS as the data operands of phase 2, one 1 KB block per
//            matrix-core instruction in lane order (no bank conflicts on either side);
//   phase 2  the wave computes its 16 output block rows for all 128 columns: 8 column tiles x
//            KK = ceil(pb / 32) contraction steps of v_mfma_f32_16x16x32_bf16, its KK operand tiles of
//            B resident in registers, the data operands read from LDS (16 bytes per lane) a few
//            instructions ahead of their use;
//   phase 3  128-point transform along the columns: three register stages, four fused DPP
//            stages, absmax; workgroup absmax through LDS;
//   phase 4  scale, round/clamp, pack; b = 4 stores dwords, b = 3 assembles the row's bytes in LDS
//            and all waves copy them out in 16-byte units.
// Column tile nt holds columns {8 c + nt}, so a lane ends up with 8 consecutive columns of 4
// block rows.  One wave per 16 block rows keeps a wave near 100 VGPRs, so two workgroups share a
// CU.  A workgroup loops over rows; barriers order the LDS reuse.
//
// Short Sylvester factors (CB < 4): n = p * 2^k with k = CB + 3 = 5 or 6 has block rows of only 32
// or 64 columns, so RPW = 128 / 2^k consecutive rows of X are laid side by side and taken in one
// pass: column group c = (row of the pass, 8-column chunk of that row).  The block product treats
// the 128 columns alike; the column transform then runs over CB lane bits only, and absmax, scale
// and the output rows are per row of the pass.  Here the block is H_p itself, of any order
// 4 <= p <= 256.
#include "wave_common.h"

namespace rq {
namespace {

// LDS operand buffer: for every (column tile nt, contraction step kk) one 1 KB block holding the data
// operand of that matrix-core instruction in lane order - lane (g, c) finds the 8 block rows
// 32 kk + 8 g .. + 7 of column (c, nt) at byte lane * 16 of the block.  A read instruction thus takes
// 1 KB of consecutive bytes and a phase-1 write instruction (8 bytes per lane: 4 block rows) 512
// consecutive bytes: neither meets a bank conflict, with no swizzle and no padding.  (Measured with a
// read-only probe on this chip: 16-byte reads in lane order move 488 bytes per ns and CU, a layout that
// gives the 16 lanes of a DPP row 16 different 16-byte slots of a 256-byte window in scattered order only
// 375.)
template <int KK>
constexpr size_t wg_ops_bytes() { return (size_t)8 * KK * 1024; }

template <int KK>
constexpr size_t wg_lds_bytes() { return wg_ops_bytes<KK>() + (size_t)KK * 32 * 48; }

// Register budget, as waves per SIMD (512 VGPRs per SIMD lane).  The hardware deals the waves of
// successive workgroups round robin over the four SIMDs, so a CU holds 4 x this many waves:
//   KK <= 3, KK == 5  6 (80 VGPRs): several small workgroups per CU, or two of 9 - 10 waves (3 of
//            which may land on one SIMD, so 96 registers would often leave room for one only);
//   KK == 4, KK >= 6   4 (128): two workgroups of up to 8 waves, or one of up to 16.
// At 128 registers there is room for the next pass's 16 load registers, so its loads are issued one
// pass ahead (right after the barrier that ends phase 1) and their latency is covered by phases
// 2 - 4.  At 80 registers the same prefetch spills, and spill reloads wait on the same counter as the
// loads: measured slower.  (Touching one byte per 128 of the next row a pass ahead, to bring it into
// the L2 cache, measured no better than the plain loads either.)
template <int KK>
constexpr int wg_waves_per_simd() { return (KK <= 3 || KK == 5) ? 6 : 4; }

// Extra arguments of the quant_error form of the kernel (QE): phases 1 - 3 are the same, phase 4
// accumulates the squared quantization error per clip ratio instead of packing codes.
struct QeArgs {
    ClipList clips;
    int n_clips;
    double* partial;      // [rows][n_clips]
};

template <int KK, int BITS, bool FULL, bool QE, int CB = 4, bool F16 = false>
__global__ __launch_bounds__(128 * KK) __attribute__((amdgpu_waves_per_eu(wg_waves_per_simd<KK>())))
void k_wg_block(WaveArgs a, int pb, QeArgs qe) {
    static_assert(CB >= 2 && CB <= 4 && (CB == 4 || !FULL), "unsupported shape");
    constexpr int RPW = 16 >> CB;                        // rows of X per pass
    constexpr int SEG = 8 << CB;                         // columns of one block row (2^k)
    constexpr bool PF = wg_waves_per_simd<KK>() == 4;    // loads run one pass ahead
    __shared__ float esum[QE ? 16 : 1][QE ? RPW : 1][QE ? RQ_MAX_CLIPS : 1];   // [wave][row of the pass][clip]
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    uint8_t* const ops = lds_raw;                        // [column tile][contraction step] x 1 KB, see wg_ops_bytes
    uint8_t* const stage = lds_raw + wg_ops_bytes<KK>(); // packed codes of the row (b = 3)
    __shared__ float wmax[16 * RPW];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;                      // ceil(pb / 16)
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;    // logical column group (8 columns)
    const int rsub = CB == 4 ? 0 : c >> CB;              // row of the pass
    const int cl = CB == 4 ? c : c & ((1 << CB) - 1);    // 8-column chunk inside that row

    u32x4 A[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) A[kk] = a.tiles[(wave * KK + kk) * 64 + lane];
    const float c1h = (float)a.c1, c1l = (float)(a.c1 - (double)c1h);
    // CB < 4: the first lane stage is the plain one, the fused ones start at the second bit
    const float flip = (__builtin_popcount(CB == 4 ? c : cl >> 1) & 1) ? -1.0f : 1.0f;
    const uint32_t sg0 = (c & 1) ? 0x80000000u : 0u;

    // phase-1 geometry: lane (g, c) loads block rows 16 wave + 4 g + t, t = 0..3, at constant
    // strides from one offset.  A group of four at or beyond pb (a multiple of 4) meets zero columns
    // of B: any in-bounds data will do, and it reads the last four real rows.
    const int r0 = 16 * wave + 4 * g;
    const int eoff0 = (r0 < pb ? r0 : pb - 4) * SEG + cl * 8;
    // phase-1 writes: the lane's block rows 16 wave + 4 g .. + 3 are one 8-byte half of the unit that
    // reader lane (2 (wave & 1) + g / 2, c) takes in contraction step wave / 2
    uint8_t* const wr0 = ops + ((((wave >> 1) * 4 + 2 * (wave & 1) + (g >> 1)) * 16 + cphys) * 16 + (g & 1) * 8);
    const uint8_t* const rd0 = ops + lane * 16;

    // Units for block rows at or beyond 16 nw are never written by phase 1 but are read by the last
    // contraction step (against zero columns of B): clear the buffer once so they hold zeros.
    for (int i = threadIdx.x; i < 8 * KK * 64; i += blockDim.x)
        reinterpret_cast<u32x4*>(ops)[i] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    u32x4 R[4];
    auto load_row = [&](int64_t row) {
        const uint16_t* xr = a.X + row * a.ld;
        if constexpr (CB == 4) {
            const RowView xv = row_view(xr, a.d);
#pragma unroll
            for (int t = 0; t < 4; ++t)
                R[t] = FULL ? load16(xr + eoff0 + t * SEG) : load_chunk(xv, eoff0 + t * SEG);
        } else {
            // the lanes of a wave read different rows: per-lane addresses, whole chunks (d % 8 == 0)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                R[t] = eoff0 + t * SEG < a.d ? load16(xr + eoff0 + t * SEG) : u32x4{0u, 0u, 0u, 0u};
        }
    };
    const int64_t n_pass = (a.rows + RPW - 1) / RPW;
    // CB == 4: one row per pass, uniform over the workgroup; otherwise the lane's own row, the
    // last row standing in (loads only) for rows beyond the end
    auto load_pass = [&](int64_t ps) {
        const int64_t r = ps * RPW + rsub;
        load_row(CB == 4 || r < a.rows ? r : a.rows - 1);
    };
    if (PF && (int64_t)blockIdx.x < n_pass) load_pass(blockIdx.x);
    for (int64_t pass = blockIdx.x; pass < n_pass; pass += gridDim.x) {
        const int64_t row = pass * RPW + rsub;
        const bool live = CB == 4 || row < a.rows;
        if (!PF) load_pass(pass);
        // ---- phase 1
#pragma unroll
        for (int ic = 0; ic < 8; ++ic) {
            const uint32_t sel = (ic & 1) ? 0x07060302u : 0x05040100u;
            uint2 v;
            v.x = __builtin_amdgcn_perm(R[1][ic >> 1], R[0][ic >> 1], sel);
            v.y = __builtin_amdgcn_perm(R[3][ic >> 1], R[2][ic >> 1], sel);
            *reinterpret_cast<uint2*>(wr0 + ic * (KK * 1024)) = v;
        }
        __syncthreads();
        if (PF && pass + gridDim.x < n_pass) load_pass(pass + gridDim.x);
        // ---- phase 2
        f32x4 acc[8];
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        {
            // The 8 KK operand reads run DEPTH ahead of the matrix-core instructions that use them, in a ring
            // of DEPTH register quads; the contraction step is the outer loop, so that consecutive
            // instructions go to different accumulators and none waits for its predecessor's result.
            // (3 where the 80-register kernels have room for it, 2 in their padded-row and quant_error forms)
            constexpr int DEPTH = KK >= 6 ? 4 : (FULL && !QE) ? 3 : 2, ITEMS = 8 * KK;
            auto read_item = [&](int i) {                // item i = (contraction step i / 8, column tile i % 8)
                return *reinterpret_cast<const u32x4*>(rd0 + ((i % 8) * KK + i / 8) * 1024);
            };
            u32x4 ring[DEPTH];
#pragma unroll
            for (int i = 0; i < DEPTH; ++i) ring[i] = read_item(i);
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                __builtin_amdgcn_sched_barrier(0);
                acc[i % 8] = mfma_pm1<F16>(A[i / 8], ring[i % DEPTH], acc[i % 8]);
                if (i + DEPTH < ITEMS) ring[i % DEPTH] = read_item(i + DEPTH);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- phase 3
#pragma unroll
        for (int s = 1; s < 8; s <<= 1)
#pragma unroll
            for (int nt = 0; nt < 8; ++nt)
                if (!(nt & s)) {
                    const f32x4 u = acc[nt], v = acc[nt | s];
                    acc[nt] = u + v;
                    acc[nt | s] = u - v;
                }
        float m = 0.0f;
        // the stage signs are rebuilt from the column group every pass (two instructions each) rather
        // than held in registers across phases 1 and 2
        int cs = c;
        asm volatile("" : "+v"(cs));
        float sf[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) sf[b] = __uint_as_float(0x3F800000u | ((uint32_t)(cs >> b) << 31));
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            f32x4 v = acc[nt];
            if constexpr (CB == 4) {
                lane_stages_fused(v, sf[0], sf[1], sf[2], sf[3]);
            } else {
                lane_stage<kDppXor1>(v, sg0);
                lane_stages_tail<CB>(v, sf);
            }
            acc[nt] = v;
            m = absmax4(m, v);
        }
        m = wave_absmax<CB>(m);                          // over the lanes that share the row
        if (g == 0 && cl == 0) wmax[wave * RPW + rsub] = m;
        __syncthreads();    // also: every wave is done reading this row's operands from LDS
        m = wmax[rsub];
        for (int w = 1; w < nw; ++w) m = fmaxf(m, wmax[w * RPW + rsub]);
        // ---- phase 4
        if constexpr (QE) {
            float v[32];
#pragma unroll
            for (int nt = 0; nt < 8; ++nt)
#pragma unroll
                for (int ip = 0; ip < 4; ++ip) v[nt * 4 + ip] = acc[nt][ip];
            // the sums run over the lanes that share a row of the pass: CB lane bits and the four DPP rows
            qe_candidates<32, BITS, CB>(v, m, flip, qe.clips, 0, qe.n_clips, [&](int k, float e2) {
                if (g == 0 && cl == 0) esum[wave][rsub][k] = e2;
            });
            __syncthreads();   // the next row writes esum only after two more barriers
            for (int i = threadIdx.x; i < RPW * qe.n_clips; i += blockDim.x) {
                const int rs = i / qe.n_clips, k = i - rs * qe.n_clips;
                const int64_t orow = pass * RPW + rs;
                if (orow < a.rows) {
                    float t = 0.0f;
                    for (int w = 0; w < nw; ++w) t += esum[w][rs][k];
                    const double nn = (double)pb * (double)SEG;
                    qe.partial[orow * qe.n_clips + k] = (double)t / (nn * nn);
                }
            }
            continue;
        }
        // (2^b - 1) / (clip m) from a float pair of the constant: reciprocal, Newton step, correction
        const float s = m > 0.0f ? flip * div_pair(c1h, c1l, m) : 0.0f;
        uint32_t* out = a.codes + row * (int64_t)(SEG * BITS / 32) * pb;   // used by live lanes only
#pragma unroll
        for (int ip = 0; ip < 4; ++ip) {
            const int ao = 16 * wave + 4 * ip + g;      // output block row of this register
            const uint32_t w = Quant<BITS>::pack8(acc[0][ip], acc[1][ip], acc[2][ip], acc[3][ip],
                                                  acc[4][ip], acc[5][ip], acc[6][ip], acc[7][ip], s);
            if constexpr (CB == 4) {
                const int word = ao * 16 + c;
                if (BITS == 4) {
                    if (ao < pb) store_codes(out + word, w);
                } else {
                    stage24(stage, word, w);            // block rows >= pb land beyond the copied part
                }
            } else if (ao < pb) {
                // the pass's rows are staged one after the other, each pb * 2^CB groups of 8 codes
                if (BITS == 4) {
                    if (live) store_codes(out + (ao << CB) + cl, w);
                } else {
                    stage24(stage, ((rsub * pb + ao) << CB) + cl, w);
                }
            }
        }
        if (BITS == 3 && CB < 4) {
            // as below; a wave's 16 block rows are 3 * 2^CB 16-byte units in each row of the pass
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            constexpr int UPR = 3 << CB;
            const int rs = lane / UPR;
            const int unit = UPR * wave + lane % UPR;   // the row has pb * UPR / 16 units
            const int64_t orow = pass * RPW + rs;
            if (lane < 48 && unit * 16 < pb * UPR && orow < a.rows)
                __builtin_nontemporal_store(
                    *reinterpret_cast<const u32x4*>(stage + (size_t)rs * pb * UPR + unit * 16),
                    reinterpret_cast<u32x4*>(a.codes + orow * (int64_t)(SEG * 3 / 32) * pb) + unit);
        }
        if (BITS == 3 && CB == 4) {
            // a wave's 16 block rows are 768 contiguous bytes of the packed row, written and read
            // back by the same wave: no workgroup barrier, only the wave's own LDS ordering
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const int unit = 48 * wave + lane;          // 16-byte units; the row has 3 pb of them
            if (lane < 48 && unit < 3 * pb)
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(stage + unit * 16),
                                            reinterpret_cast<u32x4*>(out) + unit);
        }
        if (wave == 0 && g == 0 && cl == 0 && live) a.scales[row] = (float)(a.c2 * (double)m);
    }
}

using WgKernel = void (*)(WaveArgs, int, QeArgs);

template <int KK, int BITS, int CB, bool F16>
WgKernel pick_rq(bool full) {
    if constexpr (CB == 4) {
        return full ? static_cast<WgKernel>(k_wg_block<KK, BITS, true, false, 4, F16>)
                    : static_cast<WgKernel>(k_wg_block<KK, BITS, false, false, 4, F16>);
    } else {
        return static_cast<WgKernel>(k_wg_block<KK, BITS, false, false, CB, F16>);
    }
}

// The kernel instance for a launch, or nullptr when the combination is not built: cb = 4 needs
// KK >= 2 (smaller blocks have the one-wave kernel).
template <int KK>
WgKernel pick_kernel(int bits, bool full, bool qe, int cb, bool f16) {
    if (bits != 3 && bits != 4) return nullptr;
    if (qe && cb != 4) {
        if (cb == 3) {
            if (bits == 4) return f16 ? static_cast<WgKernel>(k_wg_block<KK, 4, false, true, 3, true>)
                                      : static_cast<WgKernel>(k_wg_block<KK, 4, false, true, 3, false>);
            return f16 ? static_cast<WgKernel>(k_wg_block<KK, 3, false, true, 3, true>)
                       : static_cast<WgKernel>(k_wg_block<KK, 3, false, true, 3, false>);
        }
        if (cb == 2) {
            if (bits == 4) return f16 ? static_cast<WgKernel>(k_wg_block<KK, 4, false, true, 2, true>)
                                      : static_cast<WgKernel>(k_wg_block<KK, 4, false, true, 2, false>);
            return f16 ? static_cast<WgKernel>(k_wg_block<KK, 3, false, true, 2, true>)
                       : static_cast<WgKernel>(k_wg_block<KK, 3, false, true, 2, false>);
        }
        return nullptr;
    }
    if (qe) {
        if constexpr (KK >= 2) {
            if (f16) {
                if (bits == 4) return full ? static_cast<WgKernel>(k_wg_block<KK, 4, true, true, 4, true>)
                                           : static_cast<WgKernel>(k_wg_block<KK, 4, false, true, 4, true>);
                return full ? static_cast<WgKernel>(k_wg_block<KK, 3, true, true, 4, true>)
                            : static_cast<WgKernel>(k_wg_block<KK, 3, false, true, 4, true>);
            }
            if (bits == 4) return full ? static_cast<WgKernel>(k_wg_block<KK, 4, true, true>)
                                       : static_cast<WgKernel>(k_wg_block<KK, 4, false, true>);
            return full ? static_cast<WgKernel>(k_wg_block<KK, 3, true, true>)
                        : static_cast<WgKernel>(k_wg_block<KK, 3, false, true>);
        }
        return nullptr;
    }
    if (cb == 4) {
        if constexpr (KK >= 2) {
            if (bits == 4) return f16 ? pick_rq<KK, 4, 4, true>(full) : pick_rq<KK, 4, 4, false>(full);
            return f16 ? pick_rq<KK, 3, 4, true>(full) : pick_rq<KK, 3, 4, false>(full);
        }
        return nullptr;
    }
    if (cb == 3) {
        if (bits == 4) return f16 ? pick_rq<KK, 4, 3, true>(false) : pick_rq<KK, 4, 3, false>(false);
        return f16 ? pick_rq<KK, 3, 3, true>(false) : pick_rq<KK, 3, 3, false>(false);
    }
    if (cb == 2) {
        if (bits == 4) return f16 ? pick_rq<KK, 4, 2, true>(false) : pick_rq<KK, 4, 2, false>(false);
        return f16 ? pick_rq<KK, 3, 2, true>(false) : pick_rq<KK, 3, 2, false>(false);
    }
    return nullptr;
}

template <int KK>
int launch_kk(const rq_hadamard* h, const WaveArgs& a, int bits, int pb, int cb, hipStream_t s,
              const QeArgs* qe = nullptr) {
    const size_t lds = wg_lds_bytes<KK>();
    const int nw = (pb + 15) / 16;
    int per_cu = (int)((size_t)h->max_lds / (lds + 128));
    const int by_waves = 4 * wg_waves_per_simd<KK>() / nw;   // see the register budget note at the kernel
    if (per_cu > by_waves) per_cu = by_waves;
    if (per_cu < 1) per_cu = 1;
    const int64_t cap = (int64_t)h->num_cu * per_cu;
    const int rpw = 16 >> cb;
    const int64_t passes = (a.rows + rpw - 1) / rpw;
    const unsigned grid = (unsigned)(passes < cap ? passes : cap);
    const bool full = cb == 4 && a.d == 128 * pb;
    WgKernel fn = pick_kernel<KK>(bits, full, qe != nullptr, cb, a.f16);
    if (!fn) return RQ_ERR_NO_ORDER;
    QeArgs q;
    if (qe) {
        q = *qe;
    } else {
        q.n_clips = 0;
        q.partial = nullptr;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(64 * nw), lds, s, a, pb, q);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int KK>
bool prepare_kk() {
    const int lds = (int)wg_lds_bytes<KK>();
    if (lds <= 48 * 1024) return true;
    for (int bits = 3; bits <= 4; ++bits)
        for (int full = 0; full < 2; ++full)
            for (int qe = 0; qe < 2; ++qe)
                for (int cb = 2; cb <= 4; ++cb)
                    for (int f16 = 0; f16 < 2; ++f16) {
                        WgKernel fn = pick_kernel<KK>(bits, full != 0, qe != 0, cb, f16 != 0);
                        if (fn && hipFuncSetAttribute(reinterpret_cast<const void*>(fn),
                                                      hipFuncAttributeMaxDynamicSharedMemorySize,
                                                      lds) != hipSuccess)
                            return false;
                    }
    return true;
}

}  // namespace

// Operand tiles of the zero-padded block `bm` (order pb): [wave][kk][lane] x 16 bytes, wave <
// ceil(pb/16), kk < ceil(pb/32); operand lane (gA, mm) of (wave, kk) holds block row
// 16 wave + 4 (mm & 3) + (mm >> 2) at the contraction slots a = 32 kk + 8 gA + i.
std::vector<uint32_t> wg_block_tiles(const std::vector<int8_t>& bm, int pb) {
    const int NW = (pb + 15) / 16, KK = (pb + 31) / 32;
    std::vector<uint32_t> t((size_t)NW * KK * 64 * 4, 0u);
    for (int w = 0; w < NW; ++w)
        for (int kk = 0; kk < KK; ++kk)
            for (int lane = 0; lane < 64; ++lane) {
                const int gA = lane >> 4, mm = lane & 15;
                const int ao = 16 * w + 4 * (mm & 3) + (mm >> 2);
                for (int i = 0; i < 8; ++i) {
                    const int ai = 32 * kk + 8 * gA + i;
                    uint32_t v = 0;
                    if (ao < pb && ai < pb) v = bm[(size_t)ao * pb + ai] > 0 ? 0x3F80u : 0xBF80u;
                    t[(((size_t)w * KK + kk) * 64 + lane) * 4 + (i >> 1)] |= v << ((i & 1) * 16);
                }
            }
    return t;
}

bool wg_block_prepare(int pb) {
    switch ((pb + 31) / 32) {
        case 1: return prepare_kk<1>();
        case 2: return prepare_kk<2>();
        case 3: return prepare_kk<3>();
        case 4: return prepare_kk<4>();
        case 5: return prepare_kk<5>();
        case 6: return prepare_kk<6>();
        case 7: return prepare_kk<7>();
        case 8: return prepare_kk<8>();
        default: return false;
    }
}

// Shape of a launch: block order and lane bits of the column transform (4: block rows of 128
// columns; 3, 2: block rows of 64 / 32 columns, several rows of X per pass).  False when the order
// is not served by this kernel.
static bool wg_shape(const RowArgs& a, int* pb, int* cb) {
    if (a.p == 1) {
        // Sylvester orders beyond the one-wave kernel (2^14, 2^15): the block is H_128 / H_256 itself
        if (a.log2m < 14 || a.log2m > 15) return false;
        *pb = 1 << (a.log2m - 7);
        *cb = 4;
        return true;
    }
    if (a.log2m >= 7) {
        *pb = a.p << (a.log2m - 7);
        *cb = 4;
        return *pb > 32 && *pb <= 256;
    }
    *pb = a.p;
    *cb = a.log2m - 3;
    return a.log2m >= 5 && a.p >= 4 && a.p <= 256;
}

bool wg_block_supports(const rq_hadamard* h, const RowArgs& a, bool quant_error) {
    (void)quant_error;                                  // both forms cover the same shapes
    int pb, cb;
    if (h->device < 0 || !h->d_tiles || !h->wg_ok || !wg_shape(a, &pb, &cb)) return false;
    if (a.dtype != RQ_BF16 && !(a.dtype == RQ_F16 && h->d_tiles_f16)) return false;
    if ((reinterpret_cast<uintptr_t>(a.X) & 15) != 0 || (a.ld & 7) != 0 || (a.d & 7) != 0) return false;
    return true;
}

template <typename... Extra>
static int launch_by_kk(const rq_hadamard* h, const WaveArgs& w, int bits, int pb, int cb, hipStream_t s,
                        Extra... extra) {
    switch ((pb + 31) / 32) {
        case 1: return launch_kk<1>(h, w, bits, pb, cb, s, extra...);
        case 2: return launch_kk<2>(h, w, bits, pb, cb, s, extra...);
        case 3: return launch_kk<3>(h, w, bits, pb, cb, s, extra...);
        case 4: return launch_kk<4>(h, w, bits, pb, cb, s, extra...);
        case 5: return launch_kk<5>(h, w, bits, pb, cb, s, extra...);
        case 6: return launch_kk<6>(h, w, bits, pb, cb, s, extra...);
        case 7: return launch_kk<7>(h, w, bits, pb, cb, s, extra...);
        case 8: return launch_kk<8>(h, w, bits, pb, cb, s, extra...);
        default: return RQ_ERR_NO_ORDER;
    }
}

int wg_block_quant_error(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                         double* partial, hipStream_t s) {
    int pb, cb;
    if (!wg_shape(a, &pb, &cb)) return RQ_ERR_NO_ORDER;
    const bool f16 = a.dtype == RQ_F16;
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(f16 ? h->d_tiles_f16 : h->d_tiles), nullptr, nullptr, 0.0, 0.0};
    w.f16 = f16;
    QeArgs qe;
    qe.clips = clips;
    qe.n_clips = n_clips;
    qe.partial = partial;
    return launch_by_kk(h, w, a.bits, pb, cb, s, &qe);
}

int wg_block_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                             float* scales, hipStream_t s) {
    int pb, cb;
    if (!wg_shape(a, &pb, &cb)) return RQ_ERR_NO_ORDER;
    const bool f16 = a.dtype == RQ_F16;
    const double lvl = (double)((1 << a.bits) - 1);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(f16 ? h->d_tiles_f16 : h->d_tiles), codes, scales,
               lvl / (double)clip, (double)clip / (std::sqrt((double)a.n) * lvl)};
    w.f16 = f16;
    return launch_by_kk(h, w, a.bits, pb, cb, s);
}

}  // namespace rq
