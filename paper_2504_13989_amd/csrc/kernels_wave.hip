// Wave-per-row rotate-and-quantize kernels for bf16 rows and Sylvester orders 128 .. 8192.
//
// One 64-lane wave owns a row (or 16 >> CB short rows).  Per row (paper sections in brackets):
//   1. coalesced 16-byte loads, zero beyond d                         [4.2, Eq. 2]
//   2. five butterfly stages at once as a +-1 32x32 product on the matrix cores, straight
//      from the bf16 registers (exact products, fp32 accumulation)   [2.3.2, Eq. 1]
//   3. the remaining stages on the vector ALU: across registers, then across lanes with
//      DPP row permutations                                           [2.3.2, Eq. 1]
//   4. absmax (wave reduction), scale, round/clamp, bit-pack, store   [2.1, 3.1]
//
// Index layout.  An element index j of the row splits into
//   [ t | g | c | i ]   i: 3 bits inside a 16-byte chunk, c: CB bits (lane, within a 16-lane DPP
//                       row), g: 2 bits (which DPP row), t: log2(T) bits (which load)
// The matrix-core product transforms the (g, i) bits, register butterflies the t bits, DPP
// butterflies the c bits.  The transform is in place: an output index has the same layout, so
// a lane ends up holding 8 consecutive codes per load - whole dwords for b = 4, 3 bytes for
// b = 3 (merged into dwords inside each quad of lanes).
//
// DPP stages use xor-1, xor-2 (quad_perm), half-row mirror (xor-7) and a rotation by 8 (xor-8),
// each a single DPP-modified add.  With the mirror, a lane's logical column index is its lane
// number with the two low bits complemented when bit 2 is set.
#include <type_traits>

#include "wave_common.h"

namespace rq {
namespace {

// Long rows: n = 512 T (T = 2 .. 16), one wave per row.  FULL: d == n (no zero padding).
template <int T, int BITS, bool FULL, bool F16 = false>
__global__ __launch_bounds__(64) void k_wave_sylvester(WaveArgs a) {
    constexpr int ROW_DWORDS = 512 * T * BITS / 32;
    __shared__ __attribute__((aligned(16))) uint8_t stage[BITS == 3 ? ROW_DWORDS * 4 : 16];
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;    // logical column index
    const int chunk = (g << 4) + c;                     // 16-byte chunk inside a 1 KB load segment

    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;

    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const uint16_t* xr = a.X + row * a.ld;
        const RowView xv = row_view(xr, a.d);
        f32x4 acc[T][2];
        // every load of the row is issued before anything waits for one (left to itself the compiler
        // holds half of them back until the first has returned: a second memory round trip per row)
        u32x4 raw[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int e0 = (t * 64 + chunk) * 8;
            raw[t] = FULL ? load16(xr + e0) : load_chunk(xv, e0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            acc[t][0] = mfma_pm1<F16>(A0, raw[t], z);
            acc[t][1] = mfma_pm1<F16>(A1, raw[t], z);
        }
        // register stages over the t bits
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
        // lane stages over the c bits, and the running absmax
        float m = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 v = acc[t][h];
                lane_stages_fused(v, sf[0], sf[1], sf[2], sf[3]);
                acc[t][h] = v;
                m = absmax4(m, v);
            }
        m = wave_absmax<4>(m);
        const float s = m > 0.0f ? flip * (float)(a.c1 / (double)m) : 0.0f;

        uint32_t* out = a.codes + row * (int64_t)ROW_DWORDS;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const uint32_t w = Quant<BITS>::pack8(acc[t][0][0], acc[t][0][1], acc[t][0][2], acc[t][0][3],
                                                  acc[t][1][0], acc[t][1][1], acc[t][1][2], acc[t][1][3], s);
            const int word = t * 64 + chunk;            // 8-element group index inside the row
            if (BITS == 4)
                store_codes(out + word, w);
            else
                stage24(stage, word, w);
        }
        if (BITS == 3) {
            __syncthreads();
            copy_out16<ROW_DWORDS / 4>(stage, out, ROW_DWORDS / 4, lane);
            __syncthreads();
        }
        if (lane == 0) a.scales[row] = (float)(a.c2 * (double)m);
    }
}

// Few long rows: the same transform with a row split over S waves of one workgroup, so that a
// launch of a few thousand rows has enough waves to cover memory latency and a short tail.
// H_n = H_S (x) H_{n/S} (section 2.3.2, Eq. 1): output segment s is H_{n/S} applied to
// sum_s' H_S[s][s'] x_seg[s'], and that signed sum costs nothing on the matrix cores - the
// products of all S input segments accumulate into one accumulator, with the negated operand
// tile where H_S has -1.  Every wave therefore loads the whole row (S times the L1 traffic, the
// same HBM traffic) but carries only T / S accumulator sets through the vector-ALU stages; the
// waves exchange nothing but their absmax.
template <int T, int BITS, bool FULL, int S, bool F16 = false>
__global__ __launch_bounds__(64 * S) void k_wave_sylvester_split(WaveArgs a) {
    static_assert(T % S == 0 && (S == 2 || S == 4), "unsupported split");
    constexpr int TS = T / S;
    constexpr int ROW_DWORDS = 512 * T * BITS / 32;
    constexpr int SEG_DWORDS = ROW_DWORDS / S;
    __shared__ __attribute__((aligned(16))) uint8_t stage_all[BITS == 3 ? ROW_DWORDS * 4 : 16];
    __shared__ float wmax[S];
    const int lane = threadIdx.x & 63;
    const int seg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;
    const int chunk = (g << 4) + c;

    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    // operand tiles per input segment: negated where H_S[seg][sp] = -1 (Sylvester sign; bit 15 is the
    // sign of a bf16 and of an fp16 alike)
    u32x4 P0[S], P1[S];
#pragma unroll
    for (int sp = 0; sp < S; ++sp) {
        const uint32_t sg = (__builtin_popcount(seg & sp) & 1) ? 0x80008000u : 0u;
        const u32x4 sgn = {sg, sg, sg, sg};
        P0[sp] = A0 ^ sgn;
        P1[sp] = A1 ^ sgn;
    }
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;

    const int64_t row = blockIdx.x;
    if (row >= a.rows) return;                           // whole workgroup: no barrier is skipped
    const uint16_t* xr = a.X + row * a.ld;
    const RowView xv = row_view(xr, a.d);
    f32x4 acc[TS][2];
    // all T loads of the row first (see k_wave_sylvester); plain (cached) loads: the S waves of the
    // workgroup read the same lines
    u32x4 raw[TS][S];
#pragma unroll
    for (int t = 0; t < TS; ++t)
#pragma unroll
        for (int sp = 0; sp < S; ++sp) {
            const int e0 = ((sp * TS + t) * 64 + chunk) * 8;
            raw[t][sp] = FULL ? *reinterpret_cast<const u32x4*>(xr + e0) : load_chunk(xv, e0);
        }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < TS; ++t) {
        acc[t][0] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sp = 0; sp < S; ++sp) {
            acc[t][0] = mfma_pm1<F16>(P0[sp], raw[t][sp], acc[t][0]);
            acc[t][1] = mfma_pm1<F16>(P1[sp], raw[t][sp], acc[t][1]);
        }
    }
#pragma unroll
    for (int s = 1; s < TS; s <<= 1)
#pragma unroll
        for (int t = 0; t < TS; ++t)
            if (!(t & s))
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const f32x4 u = acc[t][h], v = acc[t | s][h];
                    acc[t][h] = u + v;
                    acc[t | s][h] = u - v;
                }
    float m = 0.0f;
#pragma unroll
    for (int t = 0; t < TS; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f32x4 v = acc[t][h];
            if (TS == 1) {                               // straight from the matrix cores: see lane_stages_tail
                const uint32_t sg0 = (c & 1) ? 0x80000000u : 0u;
                lane_stage<kDppXor1>(v, sg0);
                lane_stages_tail<4>(v, sf);
            } else {
                lane_stages_fused(v, sf[0], sf[1], sf[2], sf[3]);
            }
            acc[t][h] = v;
            m = absmax4(m, v);
        }
    m = wave_absmax<4>(m);
    if (lane == 0) wmax[seg] = m;
    __syncthreads();
    m = wmax[0];
#pragma unroll
    for (int w = 1; w < S; ++w) m = __builtin_fmaxf(m, wmax[w]);
    const float fl = TS == 1 ? ((__builtin_popcount(c >> 1) & 1) ? -1.0f : 1.0f) : flip;
    const float s = m > 0.0f ? fl * (float)(a.c1 / (double)m) : 0.0f;

    uint32_t* out = a.codes + row * (int64_t)ROW_DWORDS + seg * SEG_DWORDS;
    uint8_t* stage = stage_all + (BITS == 3 ? seg * SEG_DWORDS * 4 : 0);
#pragma unroll
    for (int t = 0; t < TS; ++t) {
        const uint32_t w = Quant<BITS>::pack8(acc[t][0][0], acc[t][0][1], acc[t][0][2], acc[t][0][3],
                                              acc[t][1][0], acc[t][1][1], acc[t][1][2], acc[t][1][3], s);
        const int word = t * 64 + chunk;
        if (BITS == 4)
            store_codes(out + word, w);
        else
            stage24(stage, word, w);
    }
    if (BITS == 3) {
        // the segment's bytes are written and read back by this wave only
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        copy_out16<SEG_DWORDS / 4>(stage, out, SEG_DWORDS / 4, lane);
    }
    if (threadIdx.x == 0) a.scales[row] = (float)(a.c2 * (double)m);
}

// Short rows: n = 32 << CB (128, 256, 512), 16 >> CB rows per wave pass, U passes in flight.
// Lane (g, r, c): DPP row g holds contraction slots, r selects the row of the pass, c the
// column chunk; the matrix cores transform the (g, i) bits, CB DPP stages the c bits.
// GUARD: the super-group may be ragged (rows missing at the end) or d < n.
// The vector ALU is what these kernels are bound by (about ten instructions per value), so the work that
// is per row rather than per value is done once for four passes at a time: the lane maxima of four
// passes cross the four DPP rows together (the row-swap instructions work on two registers at once) and
// leave pass k's maximum in DPP row k; that row alone forms the row's scale and multiplier (one
// division sequence for four passes) and stores the scale (one store of 16 floats for four passes);
// three more swaps hand the four multipliers back to every lane.  The codes go out through the
// iteration's base address in scalar registers plus one per-lane byte offset computed once.
//
// v_permlane16_swap(a, b) leaves a = [a0 b0 a2 b2], b = [a1 b1 a3 b3] (DPP rows of the old a, b);
// v_permlane32_swap(a, b) leaves a = [a0 a1 b0 b1], b = [a2 a3 b2 b3].
__device__ __forceinline__ void swap16(uint32_t& x, uint32_t& y) {
    const auto r = __builtin_amdgcn_permlane16_swap(x, y, false, false);
    x = r[0]; y = r[1];
}
__device__ __forceinline__ void swap32(uint32_t& x, uint32_t& y) {
    const auto r = __builtin_amdgcn_permlane32_swap(x, y, false, false);
    x = r[0]; y = r[1];
}
// Maxima of four passes over the four DPP rows: DPP row k of the result holds pass k's maximum.
// Non-negative floats are compared as unsigned patterns; SIGNED takes a float maximum (written as
// an instruction: the compiler would canonicalize operands that come out of assembly blocks first).
template <bool SIGNED = false>
__device__ __forceinline__ uint32_t max_raw(uint32_t a, uint32_t b) {
    if constexpr (SIGNED) {
        uint32_t r;
        asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
        return r;
    } else {
        return max(a, b);
    }
}
template <bool SIGNED = false>
__device__ __forceinline__ uint32_t rows_reduce4(uint32_t A, uint32_t B, uint32_t C, uint32_t D) {
    swap16(A, B);
    uint32_t x = max_raw<SIGNED>(A, B);           // [A01 B01 A23 B23]
    swap16(C, D);
    uint32_t y = max_raw<SIGNED>(C, D);           // [C01 D01 C23 D23]
    swap32(x, y);                                 // x = [A01 B01 C01 D01], y = [A23 B23 C23 D23]
    return max_raw<SIGNED>(x, y);
}
// Float maximum of two values at once over the four lanes of a quad (DPP-fused).
__device__ __forceinline__ void quad_max_pair(float& a, float& b) {
    asm("s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 3"
        : "+v"(a), "+v"(b));
}
// The reverse: out[k] = the value DPP row k holds, in every lane (same position inside the row).
__device__ __forceinline__ void rows_bcast4(uint32_t z, uint32_t (&out)[4]) {
    uint32_t z2 = z;
    swap16(z, z2);                                // z = [z0 z0 z2 z2], z2 = [z1 z1 z3 z3]
    uint32_t zc = z, z2c = z2;
    swap32(z, zc);                                // z = [z0 z0 z0 z0], zc = [z2 z2 z2 z2]
    swap32(z2, z2c);
    out[0] = z; out[1] = z2; out[2] = zc; out[3] = z2c;
}

// Codes of eight values on the rows as they are (PLAIN kernels): the single-rounding fma as everywhere, plus
// the residual e = t - round(t).  Un-rotated 16-bit inputs sit on a coarse grid and land on or next to a
// rounding tie far more often than rotated values, so a value whose residual is within the window `thr` of a
// tie is retaken from the definition in fp64 (`exact`), for that value only; one test guards the eight.
template <int BITS, typename Exact>
__device__ __forceinline__ uint32_t pack8_plain(const float (&x)[8], float cen, float s, float bias, float thr,
                                                bool any_exact, uint32_t tail_xor, Exact exact) {
    float v[8], e[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float dx = x[k] - cen;
        v[k] = fmaf(dx, s, bias);
        e[k] = fmaf(dx, s, bias - v[k]);                           // t - round(t)
    }
    float emax;
    asm("v_max3_f32 %0, |%1|, |%2|, |%3|\n\t"
        "v_max3_f32 %0, %0, |%4|, |%5|\n\t"
        "v_max3_f32 %0, %0, |%6|, |%7|\n\t"
        "v_max_f32 %0, %0, |%8|"
        : "=&v"(emax)
        : "v"(e[0]), "v"(e[1]), "v"(e[2]), "v"(e[3]), "v"(e[4]), "v"(e[5]), "v"(e[6]), "v"(e[7]));
    if (!(emax <= thr) && any_exact) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (!(__builtin_fabsf(e[k]) <= thr)) v[k] = exact(x[k]);
    }
    uint32_t w = 0;
#pragma unroll
    for (int k = 7; k >= 0; --k)
        w = (w << BITS) + __float_as_uint(__builtin_amdgcn_fmed3f(v[k], Quant<BITS>::kLo, Quant<BITS>::kHi));
    return (w - Quant<BITS>::csum()) ^ tail_xor;
}

template <int CB, int BITS, int U, bool GUARD, bool ASYM, bool F16, bool PLAIN = false>
__device__ __forceinline__ void short_rows_pass(const WaveArgs& a, const uint16_t* base, uint32_t* obase,
                                                float* sbase, float* mbase, int rem, const u32x4& A0, const u32x4& A1,
                                                const float (&sf)[4], float flip, int g, int c, int rsub,
                                                int chunk,
                                                float c1h, float c1l, float c2h, float c2l) {
    constexpr int RPW = 16 >> CB;
    constexpr int ROW_DWORDS = (32 << CB) * BITS / 32;
    static_assert(U % 4 == 0, "passes are taken four at a time");
    u32x4 raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int rr = u * RPW + rsub;
        const uint16_t* p = base + (int64_t)rr * a.ld + chunk * 8;
        if (GUARD) {
            const bool in = rr < rem && chunk * 8 < a.d;
            raw[u] = load16(in ? p : base);
            if (!in) raw[u] = u32x4{0u, 0u, 0u, 0u};
        } else {
            raw[u] = load16(p);
        }
    }
    const uint32_t code_off = (uint32_t)(rsub * ROW_DWORDS + (BITS == 4 ? chunk : (chunk >> 2) * 3 + (c & 3))) * 4u;
    uint32_t* const out0 = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(obase) + code_off);
    auto store_pass = [&](int u, uint32_t w) {
        const bool live = !GUARD || u * RPW + rsub < rem;
        uint32_t* out = out0 + u * RPW * ROW_DWORDS;
        if (BITS == 4) {
            if (live) store_codes(out, w);
        } else {
            const int qpos = c & 3;
            const uint32_t dw = merge24<(CB >= 3)>(w, qpos);
            if (live && qpos < 3) store_codes(out, dw);
        }
    };
#pragma unroll
    for (int u0 = 0; u0 < U; u0 += 4) {
        f32x4 v0[4], v1[4];
        // row of the four passes that this lane's DPP row answers for, and whether this lane stores for it
        const int srow = (u0 + g) * RPW + rsub;
        const bool store_lane = c == 0 && (!GUARD || srow < rem);
        if constexpr (ASYM) {
            // one group of 128 = the whole row (section 5.1, KV cache): min / max instead of absmax
            static_assert(!ASYM || CB == 2, "asymmetric groups: rows of 128 only");
            uint32_t mxu[4], nmu[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                v0[k] = mfma_pm1<F16>(A0, raw[u0 + k], z);
                v1[k] = mfma_pm1<F16>(A1, raw[u0 + k], z);
                lane_stages_mfma<CB>(v0[k], sf);
                lane_stages_mfma<CB>(v1[k], sf);
                // the lane holds flip * y (see lane_stages_fused): its own extremes swap with the sign
                const float yv[8] = {v0[k][0], v0[k][1], v0[k][2], v0[k][3], v1[k][0], v1[k][1], v1[k][2], v1[k][3]};
                const float lo = min8(yv), hi = max8(yv);
                float mx = flip > 0.0f ? hi : -lo;
                float nm = flip > 0.0f ? -lo : hi;                    // -min
                quad_max_pair(mx, nm);                                // over the quad: the row's lanes in this DPP row
                mxu[k] = __float_as_uint(mx);
                nmu[k] = __float_as_uint(nm);
            }
            const float mx = __uint_as_float(rows_reduce4<true>(mxu[0], mxu[1], mxu[2], mxu[3]));
            const float mn = -__uint_as_float(rows_reduce4<true>(nmu[0], nmu[1], nmu[2], nmu[3]));
            // DPP row k: the group parameters of pass u0 + k
            const double r64 = (double)mx - (double)mn;           // exact
            const float rh = (float)r64, rl = (float)(r64 - (double)rh);
            const bool flat = !(rh > 0.0f);
            const float q = flat ? 0.0f : div_pair2(c1h, c1l, rh, rl);
            constexpr double kMid = (double)(1 << (BITS - 1)) / (double)((1 << BITS) - 1);
            const float cen = (float)(a.clip * fma(r64, kMid, (double)mn));
            if (store_lane) {
                sbase[srow] = rh * (float)a.c2;
                mbase[srow] = mn * (float)a.c3;
            }
            uint32_t q4[4], c4[4];
            rows_bcast4(__float_as_uint(q), q4);
            rows_bcast4(__float_as_uint(cen), c4);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float yv[8] = {v0[k][0], v0[k][1], v0[k][2], v0[k][3], v1[k][0], v1[k][1], v1[k][2], v1[k][3]};
                const float qk = __uint_as_float(q4[k]);
                const float bias = qk > 0.0f ? Quant<BITS>::kBias : Quant<BITS>::kMagic;   // a flat group: code 0
                store_pass(u0 + k, Quant<BITS>::pack8u(yv, flip * __uint_as_float(c4[k]), flip * qk, bias));
            }
        } else {
            uint32_t mu[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                v0[k] = mfma_pm1<F16>(A0, raw[u0 + k], z);
                v1[k] = mfma_pm1<F16>(A1, raw[u0 + k], z);
                if constexpr (!PLAIN) {
                    lane_stages_mfma<CB>(v0[k], sf);
                    lane_stages_mfma<CB>(v1[k], sf);
                }
                uint32_t m = __float_as_uint(absmax4(absmax4(0.0f, v0[k]), v1[k]));
                // inside the DPP row: the lanes that share the row (CB lane bits)
                m = max(m, dpp_u<kDppXor1>(m));
                m = max(m, dpp_u<kDppXor2>(m));
                if (CB >= 3) m = max(m, dpp_u<kDppHalfMirror>(m));
                if (CB >= 4) m = max(m, dpp_u<kDppRor8>(m));
                mu[k] = m;
            }
            // DPP row k: absmax, scale and multiplier of pass u0 + k
            const float m = __uint_as_float(rows_reduce4(mu[0], mu[1], mu[2], mu[3]));
            const float qd = div_pair(c1h, c1l, m);
            const float q = m > 0.0f ? qd : 0.0f;
            if (store_lane) sbase[srow] = fmaf(m, c2l, m * c2h);
            uint32_t q4[4];
            rows_bcast4(__float_as_uint(q), q4);
            if constexpr (PLAIN) {
                uint32_t m4[4];
                rows_bcast4(__float_as_uint(m), m4);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float yv[8] = {v0[k][0], v0[k][1], v0[k][2], v0[k][3], v1[k][0], v1[k][1], v1[k][2], v1[k][3]};
                    const float qk = __uint_as_float(q4[k]), mk = __uint_as_float(m4[k]);
                    // (no window where the multiplier overflows: fp64 throughout)
                    const float thr = (mk < 4e37f && qk < 1e30f) ? 0.49998f : -1.0f;
                    constexpr double kL = (double)((1 << BITS) - 1);
                    constexpr float kQmin = -(float)(1 << (BITS - 1)), kQmax = (float)((1 << (BITS - 1)) - 1);
                    const uint32_t w = pack8_plain<BITS>(yv, 0.0f, qk, Quant<BITS>::kBias, thr, mk > 0.0f, Quant<BITS>::msb(), [&](float x) {
                        float m_here = mk;
                        asm volatile("" : "+v"(m_here));              // keeps the fp64 work inside the branch
                        const double delta64 = a.clip * (double)m_here / kL;
                        return Quant<BITS>::kBias + fminf(fmaxf((float)rint((double)x / delta64), kQmin), kQmax);
                    });
                    store_pass(u0 + k, w);
                }
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    store_pass(u0 + k, Quant<BITS>::pack8(v0[k][0], v0[k][1], v0[k][2], v0[k][3], v1[k][0], v1[k][1], v1[k][2],
                                                          v1[k][3], flip * __uint_as_float(q4[k])));
            }
        }
    }
}

// PLAIN: the same passes on the rows as they are (rq_quantize on head rows that arrive
// rotated, sections 2.1, 5.1): the matrix cores multiply by the identity - which turns the eight 16-bit
// values of a lane into fp32 without a vector-ALU instruction - and the butterfly stages are left out.
template <int CB, int BITS, int U, bool ASYM = false, bool F16 = false, bool PLAIN = false>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(U == 8 && !PLAIN ? 4 : 1)))   // 128 registers
void k_wave_short(WaveArgs a) {
    static_assert(!(PLAIN && ASYM), "the rotation-free group quantizer has a kernel of its own");
    static_assert(CB >= 2 && CB <= 4, "unsupported shape");
    constexpr int RPW = 16 >> CB;
    constexpr int N = 32 << CB;
    constexpr int ROW_DWORDS = N * BITS / 32;
    constexpr int SUPER = RPW * U;                      // rows per wave iteration
    const int lane = threadIdx.x;
    const int g = lane >> 4, nnl = lane & 15;
    const int cphys = nnl & ((1 << CB) - 1);
    const int rsub = nnl >> CB;
    const int c = (CB >= 3 && (cphys & 4)) ? (cphys ^ 3) : cphys;
    const int chunk = (g << CB) + c;
    u32x4 A0, A1;
    if constexpr (PLAIN) {
        // identity as two operand tiles: output row mm = 4 go + io of half hh is contraction slot (go, 4 hh + io),
        // so a lane gets its own eight values back in order; operand lane (gA, mm) holds slots (gA, 0 .. 7)
        const int gA = lane >> 4, mm = lane & 15;
        const uint32_t one = F16 ? 0x3C00u : 0x3F80u;
        A0 = u32x4{0u, 0u, 0u, 0u};
        A1 = u32x4{0u, 0u, 0u, 0u};
        if (gA == (mm >> 2)) {
            const int io = mm & 3;                                  // slot io (tile 0) / 4 + io (tile 1)
            A0[io >> 1] = one << ((io & 1) * 16);
            A1[2 + (io >> 1)] = one << ((io & 1) * 16);
        }
    } else {
        A0 = a.tiles[lane];
        A1 = a.tiles[64 + lane];
    }
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = PLAIN ? 1.0f : (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;     // all stages are the fused ones
    const float c1h = (float)a.c1, c1l = (float)(a.c1 - (double)c1h);
    const float c2h = (float)a.c2, c2l = (float)(a.c2 - (double)c2h);
    const bool full_d = a.d == N;

    const int64_t n_super = (a.rows + SUPER - 1) / SUPER;
    for (int64_t sgi = blockIdx.x; sgi < n_super; sgi += gridDim.x) {
        const int64_t row0 = sgi * SUPER;
        const int64_t left = a.rows - row0;
        const int rem = left < SUPER ? (int)left : SUPER;
        const uint16_t* base = a.X + row0 * a.ld;
        uint32_t* obase = a.codes + row0 * ROW_DWORDS;
        float* sbase = a.scales + row0;
        float* mbase = ASYM ? a.mins + row0 : nullptr;
        if (rem == SUPER && full_d)
            short_rows_pass<CB, BITS, U, false, ASYM, F16, PLAIN>(a, base, obase, sbase, mbase, rem, A0, A1, sf, flip, g, c, rsub, chunk,
                                                       c1h, c1l, c2h, c2l);
        else
            short_rows_pass<CB, BITS, U, true, ASYM, F16, PLAIN>(a, base, obase, sbase, mbase, rem, A0, A1, sf, flip, g, c, rsub, chunk,
                                                      c1h, c1l, c2h, c2l);
    }
}

// ---------------------------------------------------------------------------------------------
// Block kernel: n = PB * 128 with a +-1 block of order PB <= 32 along the strided axis
// (H_n = B (x) H_128, B = H_p (x) H_{2^(k-7)}; sections 2.3.2, 2.3.3).  Index layout [ a | c | i ]:
// a = block row (stride 128 elements), c = 4 lane bits, i = 3 bits inside a 16-byte chunk.
// Lane (g, c) loads the chunks of block rows a = 8 g + t, t = 0..7.  The matrix cores contract
// over a, so the eight values a lane holds for one column are first gathered from the eight
// loads into one operand (a 16-bit transpose inside the lane, v_perm_b32).  Outputs come back
// with 8 block rows x 8 consecutive columns per lane; butterflies over i (registers) and c
// (DPP), quantization and packing then work exactly as in the Sylvester kernel.
// The rotation of one row for the block kernels: loads, block product on the matrix cores, the
// 128-point transform along the columns.  y[column i][j]: register j = 4 h + ip holds block rows
// 4 j .. 4 j + 3 (one per DPP row g); only the NV = ceil(pb / 4) registers that hold real block rows
// are carried.  Values carry the lane's flip sign (see lane_stages_fused).  Returns the row's absmax.
template <bool FULL, int NV, bool F16 = false>
__device__ __forceinline__ float block_rotate_row(const WaveArgs& a, int64_t row, int e_base, const u32x4& A0,
                                              const u32x4& A1, const float (&sf)[4], float (&y)[8][NV]) {
    constexpr int NH1 = NV > 4 ? NV - 4 : 0;              // live registers of the second half
    constexpr int NH0 = NV > 4 ? 4 : NV;
    const uint16_t* xr = a.X + row * a.ld + e_base;
    const RowView xv = row_view(a.X + row * a.ld, a.d);
    u32x4 R[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
        R[t] = FULL ? load16(xr + t * 128) : load_chunk(xv, e_base + t * 128);
#pragma unroll
    for (int ic = 0; ic < 8; ++ic) {
        u32x4 bm;
        const uint32_t sel = (ic & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            bm[w] = __builtin_amdgcn_perm(R[2 * w + 1][ic >> 1], R[2 * w][ic >> 1], sel);
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        const f32x4 d0 = mfma_pm1<F16>(A0, bm, z);
#pragma unroll
        for (int j = 0; j < NH0; ++j) y[ic][j] = d0[j];
        if constexpr (NH1 > 0) {
            const f32x4 d1 = mfma_pm1<F16>(A1, bm, z);
#pragma unroll
            for (int j = 0; j < NH1; ++j) y[ic][4 + j] = d1[j];
        }
    }
#pragma unroll
    for (int s = 1; s < 8; s <<= 1)
#pragma unroll
        for (int ic = 0; ic < 8; ++ic)
            if (!(ic & s))
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    const float u = y[ic][j], v = y[ic | s][j];
                    y[ic][j] = u + v;
                    y[ic | s][j] = u - v;
                }
    float m = 0.0f;
#pragma unroll
    for (int ic = 0; ic < 8; ++ic) {
        fused_group<NH0>(&y[ic][0], sf);
        if constexpr (NH1 > 0) fused_group<NH1>(&y[ic][4], sf);
#pragma unroll
        for (int j = 0; j < NV; ++j) m = __builtin_fmaxf(m, __builtin_fabsf(y[ic][j]));
    }
    return wave_absmax<4>(m);
}

template <int BITS, bool FULL, int NV, bool F16 = false>
__global__ __launch_bounds__(64) void k_wave_block(WaveArgs a, int pb) {
    constexpr int ROW_DWORDS_PER_A = 128 * BITS / 32;
    __shared__ __attribute__((aligned(16))) uint8_t stage[BITS == 3 ? 32 * 48 : 16];
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;     // logical column chunk
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;

    // DPP row g loads the 8 block rows base_g .. base_g + 7, base_g = min(8 g, pb - 8): always inside
    // the row, at constant offsets from one address.  Where that overlaps the rows of g - 1 the
    // block operand has zero columns, so the duplicates contribute nothing.
    const int base_g = 8 * g < pb - 8 ? 8 * g : pb - 8;
    const int e_base = base_g * 128 + c * 8;
    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        float y[8][NV];
        float m = block_rotate_row<FULL, NV, F16>(a, row, e_base, A0, A1, sf, y);
        const float s = m > 0.0f ? flip * (float)(a.c1 / (double)m) : 0.0f;
        const float scale = (float)(a.c2 * (double)m);

        uint32_t* out = a.codes + row * (int64_t)(ROW_DWORDS_PER_A * pb);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int ao = 4 * j + g;                      // output block row of this register
            const uint32_t w = Quant<BITS>::pack8(y[0][j], y[1][j], y[2][j], y[3][j], y[4][j], y[5][j],
                                                  y[6][j], y[7][j], s);
            const int word = ao * 16 + c;
            if (BITS == 4) {
                if (ao < pb) store_codes(out + word, w);
            } else {
                stage24(stage, word, w);                   // block rows >= pb land beyond the copied part
            }
        }
        if (BITS == 3) {
            __syncthreads();
            copy_out16<32 * 3>(stage, out, pb * 3, lane);
            __syncthreads();
        }
        if (lane == 0) a.scales[row] = scale;
    }
}

// Rotation alone for the same block orders (rq_rotate: the online rotation of a tensor that is not
// quantized, offline weight fusion, the inverse rotation with the transposed block's operand tiles):
// the row's rotation as above, then one multiply and a 16-byte store per lane and block row (bf16 / fp16);
// fp32 results pass through LDS so that a store instruction covers 1 KB of consecutive bytes
// (store_block_f32).
struct BlockRotArgs {
    void* Y;
    int d_out;
    int64_t ld_out;
    float inv;            // 1 / sqrt(n)
};

template <bool FULL, int NV, bool F16, int OUT>
__global__ __launch_bounds__(64) void k_wave_block_rotate(WaveArgs a, int pb, BlockRotArgs o) {
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;
    __shared__ __attribute__((aligned(16))) float lds_out[OUT == 1 ? 512 : 4];   // fp32 results pass through LDS, see store_block_f32
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float k = ((__builtin_popcount(c) & 1) ? -1.0f : 1.0f) * o.inv;
    const int base_g = 8 * g < pb - 8 ? 8 * g : pb - 8;
    const int e_base = base_g * 128 + c * 8;
    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        float y[8][NV];
        (void)block_rotate_row<FULL, NV, F16>(a, row, e_base, A0, A1, sf, y);
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int ao = 4 * j + g;                      // output block row of this register
            const int col = ao * 128 + c * 8;
            const float v8[8] = {y[0][j], y[1][j], y[2][j], y[3][j], y[4][j], y[5][j], y[6][j], y[7][j]};
            if constexpr (OUT == 1) {
                // block rows 4 j .. 4 j + 3 are one block of 64 chunks: block row g, chunk c
                float* const yr = static_cast<float*>(o.Y) + row * o.ld_out + 4 * j * 128;
                store_block_f32(lds_out, g * 16 + c, lane, v8, k, 0.0f, [&](int e, const u32x4& unit) {
                    if (4 * j + (e >> 7) < pb && 4 * j * 128 + e < o.d_out)
                        __builtin_nontemporal_store(unit, reinterpret_cast<u32x4*>(yr + e));
                });
            } else if (ao < pb && col < o.d_out) {
                store8<OUT>(o.Y, row * o.ld_out + col, v8, k);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// quant_error for bf16 rows of Sylvester order n = 512 T (1024 .. 8192): the rotation of
// k_wave_sylvester, then for each clip ratio of this wave's share [k0, k1) the row's squared
// quantization error (sections 2.1, 3.1): t = y / Delta_k, r = clamp(round(t)),
// e = y - r Delta_k, sum e^2.  The grid is rows x ksplit: with few rows the candidates of one
// row are spread over several waves (each repeats the rotation) so the chip is filled.
// partial[row][k] receives sum e^2 / n^2, the row's mean squared error in the normalised domain.
template <int T, int BITS, bool F16 = false>
__global__ __launch_bounds__(64) void k_wave_quant_error(WaveArgs a, ClipList clips, int n_clips,
                                                         int ksplit, double* partial) {
    constexpr int N = 512 * T;
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;
    const int chunk = (g << 4) + c;
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;

    const int64_t n_items = a.rows * ksplit;
    for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int64_t row = item / ksplit;
        const int part = (int)(item - row * ksplit);
        const int per = (n_clips + ksplit - 1) / ksplit;
        const int k0 = part * per, k1 = (k0 + per < n_clips) ? k0 + per : n_clips;
        const RowView xv = row_view(a.X + row * a.ld, a.d);

        f32x4 acc[T][2];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const u32x4 raw = load_chunk(xv, (t * 64 + chunk) * 8);
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            acc[t][0] = mfma_pm1<F16>(A0, raw, z);
            acc[t][1] = mfma_pm1<F16>(A1, raw, z);
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
        float m = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 v = acc[t][h];
                lane_stages_fused(v, sf[0], sf[1], sf[2], sf[3]);
                acc[t][h] = v;
                m = absmax4(m, v);
            }
        m = wave_absmax(m);

        float v[T * 8];
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) v[(t * 2 + h) * 4 + i] = acc[t][h][i];
        qe_candidates<T * 8, BITS, 4>(v, m, flip, clips, k0, k1, [&](int k, float e2) {
            if (lane == 0) partial[row * n_clips + k] = (double)e2 / ((double)N * (double)N);
        });
    }
}

// The same for the block orders of k_wave_block (n = pb * 128, pb <= 32).
template <int BITS, bool FULL, int NV, bool F16 = false>
__global__ __launch_bounds__(64) void k_wave_block_qe(WaveArgs a, int pb, ClipList clips, int n_clips, int ksplit,
                                                      double* partial) {
    const int lane = threadIdx.x;
    const int g = lane >> 4, cphys = lane & 15;
    const int c = (cphys & 4) ? (cphys ^ 3) : cphys;
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const float flip = (__builtin_popcount(c) & 1) ? -1.0f : 1.0f;
    const int base_g = 8 * g < pb - 8 ? 8 * g : pb - 8;
    const int e_base = base_g * 128 + c * 8;
    const double nn = (double)pb * 128.0;
    const int64_t n_items = a.rows * ksplit;
    for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int64_t row = item / ksplit;
        const int part = (int)(item - row * ksplit);
        const int per = (n_clips + ksplit - 1) / ksplit;
        const int k0 = part * per, k1 = (k0 + per < n_clips) ? k0 + per : n_clips;
        float y[8][NV];
        const float m = block_rotate_row<FULL, NV, F16>(a, row, e_base, A0, A1, sf, y);
        float v[8 * NV];
#pragma unroll
        for (int ic = 0; ic < 8; ++ic)
#pragma unroll
            for (int j = 0; j < NV; ++j) v[ic * NV + j] = y[ic][j];
        qe_candidates<8 * NV, BITS, 4>(v, m, flip, clips, k0, k1, [&](int k, float e2) {
            if (lane == 0) partial[row * n_clips + k] = (double)e2 / (nn * nn);
        });
    }
}

// The same for short rows (n = 32 << CB: the KV head rows): 16 >> CB rows per wave pass, every
// clip ratio for every row (there are always enough rows to fill the chip).
template <int CB, int BITS, bool F16 = false>
__global__ __launch_bounds__(64) void k_wave_short_qe(WaveArgs a, ClipList clips, int n_clips, double* partial) {
    constexpr int RPW = 16 >> CB;
    constexpr int N = 32 << CB;
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
    const float flip = (__builtin_popcount(c >> 1) & 1) ? -1.0f : 1.0f;   // stages 2.. are the fused ones
    const int64_t n_pass = (a.rows + RPW - 1) / RPW;
    for (int64_t pass = blockIdx.x; pass < n_pass; pass += gridDim.x) {
        const int64_t row = pass * RPW + rsub;
        const bool live = row < a.rows;
        const bool in = live && chunk * 8 < a.d;
        u32x4 raw = load16(a.X + (in ? row * a.ld + chunk * 8 : 0));
        if (!in) raw = u32x4{0u, 0u, 0u, 0u};
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        f32x4 v0 = mfma_pm1<F16>(A0, raw, z);
        f32x4 v1 = mfma_pm1<F16>(A1, raw, z);
        lane_stage<kDppXor1>(v0, sg0);
        lane_stage<kDppXor1>(v1, sg0);
        lane_stages_tail<CB>(v0, sf);
        lane_stages_tail<CB>(v1, sf);
        float m = absmax4(absmax4(0.0f, v0), v1);
        m = wave_absmax<CB>(m);
        const float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        qe_candidates<8, BITS, CB>(v, m, flip, clips, 0, n_clips, [&](int k, float e2) {
            if (live && g == 0 && c == 0) partial[row * n_clips + k] = (double)e2 / ((double)N * (double)N);
        });
    }
}

// quant_error of the asymmetric group-128 quantizer on rows of 128 (one group per row; sections 4.1,
// 5.1): per clip ratio lo = clip min, Delta = clip (max - min) / (2^b - 1), e = (y - lo) - code Delta;
// six vector-ALU operations per value and candidate, four candidates at a time.
template <int BITS, bool F16 = false>
__global__ __launch_bounds__(64) void k_wave_short_qe_asym(WaveArgs a, ClipList clips, int n_clips, double* partial) {
    constexpr int CB = 2, RPW = 4, N = 128;
    constexpr float kL = (float)((1 << BITS) - 1);
    const int lane = threadIdx.x;
    const int g = lane >> 4, nnl = lane & 15;
    const int c = nnl & 3, rsub = nnl >> 2;
    const int chunk = (g << CB) + c;
    const u32x4 A0 = a.tiles[lane], A1 = a.tiles[64 + lane];
    float sf[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) sf[b] = ((c >> b) & 1) ? -1.0f : 1.0f;
    const uint32_t sg0 = (c & 1) ? 0x80000000u : 0u;
    const float flip = (c & 2) ? -1.0f : 1.0f;            // the one fused stage (xor-2)
    const int64_t n_pass = (a.rows + RPW - 1) / RPW;
    for (int64_t pass = blockIdx.x; pass < n_pass; pass += gridDim.x) {
        const int64_t row = pass * RPW + rsub;
        const bool live = row < a.rows;
        const bool in = live && chunk * 8 < a.d;
        u32x4 raw = load16(a.X + (in ? row * a.ld + chunk * 8 : 0));
        if (!in) raw = u32x4{0u, 0u, 0u, 0u};
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        f32x4 v0 = mfma_pm1<F16>(A0, raw, z);
        f32x4 v1 = mfma_pm1<F16>(A1, raw, z);
        lane_stage<kDppXor1>(v0, sg0);
        lane_stage<kDppXor1>(v1, sg0);
        lane_stages_tail<CB>(v0, sf);
        lane_stages_tail<CB>(v1, sf);
        const float yv[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        const float lo8 = min8(yv), hi8 = max8(yv);
        float mx = flip > 0.0f ? hi8 : -lo8;
        float nm = flip > 0.0f ? -lo8 : hi8;
        quad_rows_max_pair(mx, nm);
        const double mn64 = -(double)nm, r64 = (double)mx + (double)nm;
        const double inv_r = r64 > 0.0 ? 1.0 / r64 : 0.0;
        for (int kb = 0; kb < n_clips; kb += 4) {
            float los[4], sk[4], ndk[4], e2[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = kb + j < n_clips ? kb + j : n_clips - 1;
                // the row-independent factors (levels / clip, clip / levels) come with the clip list
                los[j] = flip * (float)((double)clips.v[k] * mn64);               // lane sign folded in
                sk[j] = flip * (float)(clips.lvl_over_clip[k] * inv_r);
                ndk[j] = -flip * (float)(clips.clip_over_lvl[k] * r64);
                e2[j] = 0.0f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float d = yv[i] - los[j];
                    const float r = __builtin_amdgcn_fmed3f(__builtin_rintf(d * sk[j]), 0.0f, kL);
                    const float e = fmaf(r, ndk[j], d);
                    e2[j] = fmaf(e, e, e2[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) e2[j] += dpp_f<kDppXor1>(e2[j]);
#pragma unroll
            for (int j = 0; j < 4; ++j) e2[j] += dpp_f<kDppXor2>(e2[j]);
#pragma unroll
            for (int j = 0; j < 4; ++j) e2[j] = rows_sum(e2[j]);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (live && g == 0 && c == 0 && kb + j < n_clips)
                    partial[row * n_clips + kb + j] = (double)e2[j] / ((double)N * (double)N);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Rotation-free quantizer (section 2.1 with the clip ratio of section 3.1 on the row itself): one
// wave per bf16 row of d <= 512 T values, the row held in registers between the absmax pass and
// the quantization pass.  Un-rotated bf16 values sit on a coarse grid, so x / Delta lands on or
// next to a rounding tie far more often than rotated values do; every code whose fp32 residual
// is within 2e-5 of a tie is therefore retaken with the exact fp64 quotient.
// The two 16-bit values of a dword as floats (exact): bf16, or IEEE fp16 when F16.
template <bool F16>
__device__ __forceinline__ float half_lo(uint32_t w) {
    if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)w);
    else return __uint_as_float(w << 16);
}
template <bool F16>
__device__ __forceinline__ float half_hi(uint32_t w) {
    if constexpr (F16) return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    else return __uint_as_float(w & 0xffff0000u);
}

struct PlainArgs {
    const uint16_t* X;
    int64_t rows;
    int d;
    int64_t ld;
    uint32_t* codes;
    float* scales;
    double clip;
    bool f16;
};

template <int T, int BITS, bool F16 = false>
__global__ __launch_bounds__(64) void k_plain_wave(PlainArgs a) {
    const int lane = threadIdx.x;
    const int nchunks = a.d >> 3;
    const int row_dwords = a.d * BITS / 32;
    constexpr double kLvl = (double)((1 << BITS) - 1);
    constexpr float kQmin = -(float)(1 << (BITS - 1)), kQmax = (float)((1 << (BITS - 1)) - 1);
    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const RowView xv = row_view(a.X + row * a.ld, a.d);
        u32x4 raw[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            raw[t] = load_chunk(xv, (t * 64 + lane) * 8);
        }
        float m = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t w = raw[t][k];
                m = __builtin_fmaxf(m, __builtin_fabsf(half_lo<F16>(w)));
                m = __builtin_fmaxf(m, __builtin_fabsf(half_hi<F16>(w)));
            }
        m = wave_absmax<4>(m);
        const double delta = a.clip * (double)m / kLvl;
        const float s = m > 0.0f ? (float)(kLvl / (a.clip * (double)m)) : 0.0f;
        uint32_t* out = a.codes + row * (int64_t)row_dwords;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int idx = t * 64 + lane;
            float x[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = half_lo<F16>(raw[t][k]);
                x[2 * k + 1] = half_hi<F16>(raw[t][k]);
            }
            uint32_t w = 0;
#pragma unroll
            for (int r = 7; r >= 0; --r) {
                float u = fmaf(x[r], s, Quant<BITS>::kBias);
                const float e = fmaf(x[r], s, Quant<BITS>::kBias - u);     // t - round(t)
                u = __builtin_amdgcn_fmed3f(u, Quant<BITS>::kLo, Quant<BITS>::kHi);
                // within 2e-5 of a rounding tie (the fp32 quotient is good to about 2e-6): the exact fp64
                // quotient decides, for this value only
                if (__builtin_fabsf(e) > 0.49998f && m > 0.0f)
                    u = Quant<BITS>::kBias + fminf(fmaxf((float)rint((double)x[r] / delta), kQmin), kQmax);
                w = (w << BITS) + __float_as_uint(u);
            }
            w = (w - Quant<BITS>::csum()) ^ Quant<BITS>::msb();
            if (BITS == 4) {
                if (idx < nchunks) store_codes(out + idx, w);
            } else {
                const int qpos = lane & 3;
                const uint32_t dw = merge24<false>(w, qpos);
                if (idx < nchunks && qpos < 3) store_codes(out + (idx >> 2) * 3 + qpos, dw);
            }
        }
        if (lane == 0) a.scales[row] = (float)delta;
    }
}

template <int T>
int launch_plain(const PlainArgs& a, int bits, hipStream_t s) {
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(a.rows < cap ? a.rows : cap);
    if (a.f16) {
        if (bits == 4) hipLaunchKernelGGL((k_plain_wave<T, 4, true>), dim3(grid), dim3(64), 0, s, a);
        else hipLaunchKernelGGL((k_plain_wave<T, 3, true>), dim3(grid), dim3(64), 0, s, a);
    } else if (bits == 4) hipLaunchKernelGGL((k_plain_wave<T, 4>), dim3(grid), dim3(64), 0, s, a);
    else hipLaunchKernelGGL((k_plain_wave<T, 3>), dim3(grid), dim3(64), 0, s, a);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <typename K>
int launch_wave(K kernel, const rq_hadamard* h, const WaveArgs& a, int64_t items, int waves_per_simd,
                hipStream_t s) {
    // one wave per item: a fresh wave starts with its loads, which hides memory latency better
    // than a resident wave looping over rows (measured); the loop only serves huge inputs
    (void)h;
    (void)waves_per_simd;
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(items < cap ? items : cap);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, a);
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int T, int S>
int launch_split(const WaveArgs& a, int bits, hipStream_t s) {
    const bool full = a.d == 512 * T;
    const dim3 grid((unsigned)a.rows), block(64 * S);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, s, a); };
    if (a.f16) {
        if (bits == 4) { if (full) go(k_wave_sylvester_split<T, 4, true, S, true>); else go(k_wave_sylvester_split<T, 4, false, S, true>); }
        else { if (full) go(k_wave_sylvester_split<T, 3, true, S, true>); else go(k_wave_sylvester_split<T, 3, false, S, true>); }
    } else {
        if (bits == 4) { if (full) go(k_wave_sylvester_split<T, 4, true, S, false>); else go(k_wave_sylvester_split<T, 4, false, S, false>); }
        else { if (full) go(k_wave_sylvester_split<T, 3, true, S, false>); else go(k_wave_sylvester_split<T, 3, false, S, false>); }
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int T>
int launch_long(const rq_hadamard* h, const WaveArgs& a, int bits, hipStream_t s) {
    // fewer rows than SIMDs: a row split over 4 (up to half the SIMDs) or 2 waves finishes sooner
    // (measured on 4096-wide rows: 64 rows 3.1 -> 2.5 us, 512 rows 4.2 -> 3.7 us, 1024 rows 4.75 -> 4.5 us;
    // from 2048 rows on one wave per row is faster)
    if constexpr (T >= 4) {
        const int64_t simds = (int64_t)h->num_cu * 4;
        const int split = h->split.load(std::memory_order_relaxed);
        if (split >= 0) {
            const int want = split > 0 ? split : (a.rows * 2 <= simds ? 4 : a.rows <= simds ? 2 : 1);
            if (want == 4) return launch_split<T, 4>(a, bits, s);
            if (want == 2) return launch_split<T, 2>(a, bits, s);
        }
    }
    const bool full = a.d == 512 * T;
    if (a.f16) {
        if (bits == 4)
            return full ? launch_wave(k_wave_sylvester<T, 4, true, true>, h, a, a.rows, 4, s)
                        : launch_wave(k_wave_sylvester<T, 4, false, true>, h, a, a.rows, 4, s);
        return full ? launch_wave(k_wave_sylvester<T, 3, true, true>, h, a, a.rows, 4, s)
                    : launch_wave(k_wave_sylvester<T, 3, false, true>, h, a, a.rows, 4, s);
    }
    if (bits == 4)
        return full ? launch_wave(k_wave_sylvester<T, 4, true>, h, a, a.rows, 4, s)
                    : launch_wave(k_wave_sylvester<T, 4, false>, h, a, a.rows, 4, s);
    return full ? launch_wave(k_wave_sylvester<T, 3, true>, h, a, a.rows, 4, s)
                : launch_wave(k_wave_sylvester<T, 3, false>, h, a, a.rows, 4, s);
}

// Passes in flight per wave: four, or eight on inputs of 2^27 elements and more, where the deeper queue of
// loads is worth 3 - 4 % (KV head rows: 4 194 304 x 128, b = 3, 230 -> 223 us, asymmetric 258 -> 248 us) and
// the longer wave no longer costs anything at the ends of the launch (65 536 rows: 5.6 -> 6.0 us).
inline bool short_deep(const WaveArgs& a, int n) { return a.rows * (int64_t)n >= ((int64_t)1 << 27); }

template <int CB, int U>
int launch_short_u(const rq_hadamard* h, const WaveArgs& a, int bits, hipStream_t s) {
    constexpr int SUPER = (16 >> CB) * U;
    const int64_t items = (a.rows + SUPER - 1) / SUPER;
    if (a.f16)
        return bits == 4 ? launch_wave(k_wave_short<CB, 4, U, false, true>, h, a, items, 8, s)
                         : launch_wave(k_wave_short<CB, 3, U, false, true>, h, a, items, 8, s);
    return bits == 4 ? launch_wave(k_wave_short<CB, 4, U>, h, a, items, 8, s)
                     : launch_wave(k_wave_short<CB, 3, U>, h, a, items, 8, s);
}

template <int CB>
int launch_short(const rq_hadamard* h, const WaveArgs& a, int bits, hipStream_t s) {
    return short_deep(a, 32 << CB) ? launch_short_u<CB, 8>(h, a, bits, s) : launch_short_u<CB, 4>(h, a, bits, s);
}

template <int U>
int launch_short_asym_u(const rq_hadamard* h, const WaveArgs& a, int bits, hipStream_t s) {
    constexpr int SUPER = 4 * U;
    const int64_t items = (a.rows + SUPER - 1) / SUPER;
    if (a.f16)
        return bits == 4 ? launch_wave(k_wave_short<2, 4, U, true, true>, h, a, items, 8, s)
                         : launch_wave(k_wave_short<2, 3, U, true, true>, h, a, items, 8, s);
    return bits == 4 ? launch_wave(k_wave_short<2, 4, U, true>, h, a, items, 8, s)
                     : launch_wave(k_wave_short<2, 3, U, true>, h, a, items, 8, s);
}

int launch_short_asym(const rq_hadamard* h, const WaveArgs& a, int bits, hipStream_t s) {
    return short_deep(a, 128) ? launch_short_asym_u<8>(h, a, bits, s) : launch_short_asym_u<4>(h, a, bits, s);
}

}  // namespace

// The +-1 32x32 block as matrix-core operands.  Operand lane (gA, mm) holds row mm of one
// 16-row half for the 8 contraction slots (gA, i).  Row mm = 4 go + io of half hh produces the
// output whose transformed bits are (go, 4 hh + io); the entry is the Sylvester sign between
// that output index and the input slot (gA, i).
std::vector<uint32_t> wave_sylvester_tiles() {
    std::vector<uint32_t> t(2 * 64 * 4, 0u);
    for (int hh = 0; hh < 2; ++hh)
        for (int lane = 0; lane < 64; ++lane) {
            const int gA = lane >> 4, mm = lane & 15, go = mm >> 2, io = mm & 3;
            const int low3 = 4 * hh + io;
            for (int i = 0; i < 8; ++i) {
                const int par = (__builtin_popcount(low3 & i) + __builtin_popcount(go & gA)) & 1;
                const uint32_t v = par ? 0xBF80u : 0x3F80u;   // bf16 -1 / +1
                t[(hh * 64 + lane) * 4 + (i >> 1)] |= v << ((i & 1) * 16);
            }
        }
    return t;
}

std::vector<uint32_t> tiles_to_f16(const std::vector<uint32_t>& t) {
    std::vector<uint32_t> o(t.size());
    for (size_t i = 0; i < t.size(); ++i) {
        uint32_t w = 0;
        for (int h = 0; h < 2; ++h) {
            const uint32_t v = (t[i] >> (16 * h)) & 0xffffu;     // 0, bf16 +1 or bf16 -1
            const uint32_t f = v == 0x3F80u ? 0x3C00u : v == 0xBF80u ? 0xBC00u : 0u;
            w |= f << (16 * h);
        }
        o[i] = w;
    }
    return o;
}

template <int NV>
static void launch_block_nv(int bits, bool full, unsigned grid, hipStream_t s, const WaveArgs& w, int pb) {
    if (w.f16) {
        if (bits == 4) {
            if (full) hipLaunchKernelGGL((k_wave_block<4, true, NV, true>), dim3(grid), dim3(64), 0, s, w, pb);
            else hipLaunchKernelGGL((k_wave_block<4, false, NV, true>), dim3(grid), dim3(64), 0, s, w, pb);
        } else {
            if (full) hipLaunchKernelGGL((k_wave_block<3, true, NV, true>), dim3(grid), dim3(64), 0, s, w, pb);
            else hipLaunchKernelGGL((k_wave_block<3, false, NV, true>), dim3(grid), dim3(64), 0, s, w, pb);
        }
        return;
    }
    if (bits == 4) {
        if (full) hipLaunchKernelGGL((k_wave_block<4, true, NV>), dim3(grid), dim3(64), 0, s, w, pb);
        else hipLaunchKernelGGL((k_wave_block<4, false, NV>), dim3(grid), dim3(64), 0, s, w, pb);
    } else {
        if (full) hipLaunchKernelGGL((k_wave_block<3, true, NV>), dim3(grid), dim3(64), 0, s, w, pb);
        else hipLaunchKernelGGL((k_wave_block<3, false, NV>), dim3(grid), dim3(64), 0, s, w, pb);
    }
}

// Matrix-core operand of a +-1 block `bm` (row-major, order 8 <= pb <= 32) for the block kernel.
// Contraction slot (gA, i) carries block row r = min(8 gA, pb - 8) + i of the input, and counts
// only where r >= 8 gA (below that it duplicates a row of the previous slot group): other
// columns are zero.  Operand lane (gA, mm) holds, for half hh, row 16 hh + 4 (mm & 3) + (mm >> 2)
// of the block.
std::vector<uint32_t> wave_block_tiles(const std::vector<int8_t>& bm, int pb) {
    std::vector<uint32_t> t(2 * 64 * 4, 0u);
    for (int hh = 0; hh < 2; ++hh)
        for (int lane = 0; lane < 64; ++lane) {
            const int gA = lane >> 4, mm = lane & 15;
            const int ao = 16 * hh + 4 * (mm & 3) + (mm >> 2);
            const int base = 8 * gA < pb - 8 ? 8 * gA : pb - 8;
            for (int i = 0; i < 8; ++i) {
                const int ai = base + i;
                uint32_t v = 0;
                if (ao < pb && ai >= 8 * gA && ai < pb) v = bm[(size_t)ao * pb + ai] > 0 ? 0x3F80u : 0xBF80u;
                t[(hh * 64 + lane) * 4 + (i >> 1)] |= v << ((i & 1) * 16);
            }
        }
    return t;
}

static bool wave_dtype_ok(const rq_hadamard* h, const RowArgs& a) {
    return a.dtype == RQ_BF16 || (a.dtype == RQ_F16 && h->d_tiles_f16);
}

bool wave_block_supports(const rq_hadamard* h, const RowArgs& a) {
    if (h->device < 0 || !h->d_tiles || !wave_dtype_ok(h, a) || a.p == 1) return false;
    if (a.log2m < 7 || (a.p << (a.log2m - 7)) > 32 || (a.p << (a.log2m - 7)) < 8) return false;
    if ((reinterpret_cast<uintptr_t>(a.X) & 15) != 0 || (a.ld & 7) != 0 || (a.d & 7) != 0) return false;
    return true;
}

int wave_block_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                               float* scales, hipStream_t s) {
    const double lvl = (double)((1 << a.bits) - 1);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(h->d_tiles), codes, scales,
               lvl / (double)clip, (double)clip / (std::sqrt((double)a.n) * lvl)};
    if (a.dtype == RQ_F16) {
        w.f16 = true;
        w.tiles = static_cast<const u32x4*>(h->d_tiles_f16);
    }
    const int pb = a.p << (a.log2m - 7);
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(a.rows < cap ? a.rows : cap);
    const bool full = a.d == a.n;
    switch ((pb + 3) / 4) {
        case 2: launch_block_nv<2>(a.bits, full, grid, s, w, pb); break;
        case 3: launch_block_nv<3>(a.bits, full, grid, s, w, pb); break;
        case 4: launch_block_nv<4>(a.bits, full, grid, s, w, pb); break;
        case 5: launch_block_nv<5>(a.bits, full, grid, s, w, pb); break;
        case 6: launch_block_nv<6>(a.bits, full, grid, s, w, pb); break;
        case 7: launch_block_nv<7>(a.bits, full, grid, s, w, pb); break;
        case 8: launch_block_nv<8>(a.bits, full, grid, s, w, pb); break;
        default: return RQ_ERR_NO_ORDER;
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int NV>
static void launch_block_rotate_nv(bool full, bool f16, int out, unsigned grid, hipStream_t s, const WaveArgs& w, int pb,
                                   const BlockRotArgs& o) {
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, w, pb, o); };
    auto pick_out = [&](auto full_c, auto f16_c) {
        constexpr bool FL = decltype(full_c)::value, FH = decltype(f16_c)::value;
        if (out == 0) go(k_wave_block_rotate<FL, NV, FH, 0>);
        else if (out == 1) go(k_wave_block_rotate<FL, NV, FH, 1>);
        else go(k_wave_block_rotate<FL, NV, FH, 2>);
    };
    if (full) {
        if (f16) pick_out(std::true_type{}, std::true_type{}); else pick_out(std::true_type{}, std::false_type{});
    } else {
        if (f16) pick_out(std::false_type{}, std::true_type{}); else pick_out(std::false_type{}, std::false_type{});
    }
}

bool wave_block_rotate_supports(const rq_hadamard* h, const RowArgs& a, int transpose, const OutArgs& o) {
    if (!wave_block_supports(h, a)) return false;
    if (transpose && (!h->d_tiles_t || (a.dtype == RQ_F16 && !h->d_tiles_t_f16))) return false;
    if ((reinterpret_cast<uintptr_t>(o.Y) & 15) != 0 || (o.d_out & 7) != 0) return false;
    return o.dtype == RQ_F32 ? (o.ld_out & 3) == 0 : (o.ld_out & 7) == 0;
}

int wave_block_rotate(const rq_hadamard* h, const RowArgs& a, int transpose, const OutArgs& o, hipStream_t s) {
    const bool f16 = a.dtype == RQ_F16;
    const void* tiles = transpose ? (f16 ? h->d_tiles_t_f16 : h->d_tiles_t) : (f16 ? h->d_tiles_f16 : h->d_tiles);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld, static_cast<const u32x4*>(tiles), nullptr, nullptr,
               0.0, 0.0};
    w.f16 = f16;
    const BlockRotArgs bo{o.Y, o.d_out, o.ld_out, (float)(1.0 / std::sqrt((double)a.n))};
    const int out = o.dtype == RQ_BF16 ? 0 : o.dtype == RQ_F32 ? 1 : 2;
    const int pb = a.p << (a.log2m - 7);
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(a.rows < cap ? a.rows : cap);
    const bool full = a.d == a.n;
    switch ((pb + 3) / 4) {
        case 2: launch_block_rotate_nv<2>(full, f16, out, grid, s, w, pb, bo); break;
        case 3: launch_block_rotate_nv<3>(full, f16, out, grid, s, w, pb, bo); break;
        case 4: launch_block_rotate_nv<4>(full, f16, out, grid, s, w, pb, bo); break;
        case 5: launch_block_rotate_nv<5>(full, f16, out, grid, s, w, pb, bo); break;
        case 6: launch_block_rotate_nv<6>(full, f16, out, grid, s, w, pb, bo); break;
        case 7: launch_block_rotate_nv<7>(full, f16, out, grid, s, w, pb, bo); break;
        case 8: launch_block_rotate_nv<8>(full, f16, out, grid, s, w, pb, bo); break;
        default: return RQ_ERR_NO_ORDER;
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

bool wave_supports(const rq_hadamard* h, const RowArgs& a) {
    if (h->device < 0 || !h->d_tiles || !wave_dtype_ok(h, a) || a.p != 1) return false;
    if (a.log2m < 7 || a.log2m > 13) return false;
    if ((reinterpret_cast<uintptr_t>(a.X) & 15) != 0 || (a.ld & 7) != 0 || (a.d & 7) != 0) return false;
    return true;
}

bool wave_quant_error_supports(const rq_hadamard* h, const RowArgs& a) {
    return wave_supports(h, a) || wave_block_supports(h, a);
}

static int qe_ksplit(const rq_hadamard* h, int64_t rows, int n_clips) {
    // Spread one row's candidates over several waves when there are few rows, aiming at about one
    // wave per SIMD: every extra wave of a row repeats the rotation (about two candidates' worth
    // of work), so splitting further than that costs more than it balances.
    const int64_t target = (int64_t)h->num_cu * 4;
    int ksplit = (int)((target + rows - 1) / rows);
    if (ksplit < 1) ksplit = 1;
    if (ksplit > n_clips) ksplit = n_clips;
    if (ksplit > 8) ksplit = 8;
    return ksplit;
}

template <int T>
static int launch_qe(const rq_hadamard* h, const WaveArgs& w, const ClipList& clips, int n_clips,
                     int bits, double* partial, hipStream_t s) {
    const int ksplit = qe_ksplit(h, w.rows, n_clips);
    const int64_t items = w.rows * ksplit;
    const int64_t cap = 1 << 24;
    const unsigned grid = (unsigned)(items < cap ? items : cap);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(grid), dim3(64), 0, s, w, clips, n_clips, ksplit, partial); };
    if (w.f16) {
        if (bits == 4) go(k_wave_quant_error<T, 4, true>); else go(k_wave_quant_error<T, 3, true>);
    } else {
        if (bits == 4) go(k_wave_quant_error<T, 4, false>); else go(k_wave_quant_error<T, 3, false>);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int NV>
static int launch_block_qe(const rq_hadamard* h, const WaveArgs& w, int pb, const ClipList& clips, int n_clips,
                           int bits, double* partial, hipStream_t s) {
    const int ksplit = qe_ksplit(h, w.rows, n_clips);
    const int64_t items = w.rows * ksplit;
    const int64_t cap = 1 << 24;
    const dim3 grid((unsigned)(items < cap ? items : cap)), block(64);
    const bool full = w.d == pb * 128;
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, s, w, pb, clips, n_clips, ksplit, partial); };
    if (w.f16) {
        if (bits == 4) { if (full) go(k_wave_block_qe<4, true, NV, true>); else go(k_wave_block_qe<4, false, NV, true>); }
        else { if (full) go(k_wave_block_qe<3, true, NV, true>); else go(k_wave_block_qe<3, false, NV, true>); }
    } else {
        if (bits == 4) { if (full) go(k_wave_block_qe<4, true, NV, false>); else go(k_wave_block_qe<4, false, NV, false>); }
        else { if (full) go(k_wave_block_qe<3, true, NV, false>); else go(k_wave_block_qe<3, false, NV, false>); }
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int CB>
static int launch_short_qe(const WaveArgs& w, const ClipList& clips, int n_clips, int bits, double* partial,
                           hipStream_t s) {
    const int64_t passes = (w.rows + (16 >> CB) - 1) / (16 >> CB);
    const int64_t cap = 1 << 24;
    const dim3 grid((unsigned)(passes < cap ? passes : cap)), block(64);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, s, w, clips, n_clips, partial); };
    if (w.f16) {
        if (bits == 4) go(k_wave_short_qe<CB, 4, true>); else go(k_wave_short_qe<CB, 3, true>);
    } else {
        if (bits == 4) go(k_wave_short_qe<CB, 4, false>); else go(k_wave_short_qe<CB, 3, false>);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int wave_quant_error_asym(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                          double* partial, hipStream_t s) {
    const bool f16 = a.dtype == RQ_F16;
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(f16 ? h->d_tiles_f16 : h->d_tiles), nullptr, nullptr, 0.0, 0.0};
    w.f16 = f16;
    const int64_t passes = (w.rows + 3) / 4;
    const int64_t cap = 1 << 24;
    const dim3 grid((unsigned)(passes < cap ? passes : cap)), block(64);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, s, w, clips, n_clips, partial); };
    if (f16) {
        if (a.bits == 4) go(k_wave_short_qe_asym<4, true>); else go(k_wave_short_qe_asym<3, true>);
    } else {
        if (a.bits == 4) go(k_wave_short_qe_asym<4, false>); else go(k_wave_short_qe_asym<3, false>);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

int wave_quant_error(const rq_hadamard* h, const RowArgs& a, const ClipList& clips, int n_clips,
                     double* partial, hipStream_t s) {
    const bool f16 = a.dtype == RQ_F16;
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(f16 ? h->d_tiles_f16 : h->d_tiles), nullptr, nullptr, 0.0, 0.0};
    w.f16 = f16;
    if (a.p > 1) {
        const int pb = a.p << (a.log2m - 7);
        switch ((pb + 3) / 4) {
            case 2: return launch_block_qe<2>(h, w, pb, clips, n_clips, a.bits, partial, s);
            case 3: return launch_block_qe<3>(h, w, pb, clips, n_clips, a.bits, partial, s);
            case 4: return launch_block_qe<4>(h, w, pb, clips, n_clips, a.bits, partial, s);
            case 5: return launch_block_qe<5>(h, w, pb, clips, n_clips, a.bits, partial, s);
            case 6: return launch_block_qe<6>(h, w, pb, clips, n_clips, a.bits, partial, s);
            case 7: return launch_block_qe<7>(h, w, pb, clips, n_clips, a.bits, partial, s);
            case 8: return launch_block_qe<8>(h, w, pb, clips, n_clips, a.bits, partial, s);
            default: return RQ_ERR_NO_ORDER;
        }
    }
    switch (a.log2m) {
        case 7: return launch_short_qe<2>(w, clips, n_clips, a.bits, partial, s);
        case 8: return launch_short_qe<3>(w, clips, n_clips, a.bits, partial, s);
        case 9: return launch_short_qe<4>(w, clips, n_clips, a.bits, partial, s);
        case 10: return launch_qe<2>(h, w, clips, n_clips, a.bits, partial, s);
        case 11: return launch_qe<4>(h, w, clips, n_clips, a.bits, partial, s);
        case 12: return launch_qe<8>(h, w, clips, n_clips, a.bits, partial, s);
        case 13: return launch_qe<16>(h, w, clips, n_clips, a.bits, partial, s);
        default: return RQ_ERR_NO_ORDER;
    }
}

int wave_rotate_quantize(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                         float* scales, hipStream_t s) {
    const double lvl = (double)((1 << a.bits) - 1);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(h->d_tiles), codes, scales,
               lvl / (double)clip, (double)clip / (std::sqrt((double)a.n) * lvl)};
    if (a.dtype == RQ_F16) {
        w.f16 = true;
        w.tiles = static_cast<const u32x4*>(h->d_tiles_f16);
    }
    switch (a.log2m) {
        case 7: return launch_short<2>(h, w, a.bits, s);
        case 8: return launch_short<3>(h, w, a.bits, s);
        case 9: return launch_short<4>(h, w, a.bits, s);
        case 10: return launch_long<2>(h, w, a.bits, s);
        case 11: return launch_long<4>(h, w, a.bits, s);
        case 12: return launch_long<8>(h, w, a.bits, s);
        case 13: return launch_long<16>(h, w, a.bits, s);
        default: return RQ_ERR_NO_ORDER;
    }
}

// Rotation-free quantizers on head rows of 128, 256 or 512 16-bit values: the short-row passes with the
// identity on the matrix cores.
template <int CB, int U>
static int launch_plain_short_u(const WaveArgs& a, int bits, hipStream_t s) {
    constexpr int SUPER = (16 >> CB) * U;
    const int64_t items = (a.rows + SUPER - 1) / SUPER;
    const int64_t cap = 1 << 24;
    const dim3 grid((unsigned)(items < cap ? items : cap)), block(64);
    auto go = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, s, a); };
    if (a.f16) {
        if (bits == 4) go(k_wave_short<CB, 4, U, false, true, true>); else go(k_wave_short<CB, 3, U, false, true, true>);
    } else {
        if (bits == 4) go(k_wave_short<CB, 4, U, false, false, true>); else go(k_wave_short<CB, 3, U, false, false, true>);
    }
    return hipGetLastError() == hipSuccess ? RQ_OK : RQ_ERR_HIP;
}

template <int CB>
static int launch_plain_short(const WaveArgs& a, int bits, hipStream_t s) {
    return short_deep(a, 32 << CB) ? launch_plain_short_u<CB, 8>(a, bits, s) : launch_plain_short_u<CB, 4>(a, bits, s);
}

bool plain_wave_short_supports(const void* X, int dtype, int d, int64_t ld) {
    return (dtype == RQ_BF16 || dtype == RQ_F16) && (d == 128 || d == 256 || d == 512) && ld % 8 == 0 &&
           (reinterpret_cast<uintptr_t>(X) % 16) == 0;
}

int plain_wave_short_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                              uint32_t* codes, float* scales, hipStream_t s) {
    const double lvl = (double)((1 << bits) - 1);
    WaveArgs w{static_cast<const uint16_t*>(X), rows, d, ld, nullptr, codes, scales, lvl / (double)clip, (double)clip / lvl};
    w.clip = (double)clip;
    w.f16 = dtype == RQ_F16;
    if (d == 128) return launch_plain_short<2>(w, bits, s);
    if (d == 256) return launch_plain_short<3>(w, bits, s);
    return launch_plain_short<4>(w, bits, s);
}

bool plain_wave_supports(const void* X, int dtype, int d, int64_t ld) {
    return (dtype == RQ_BF16 || dtype == RQ_F16) && d % 32 == 0 && d <= 512 * 40 && ld % 8 == 0 &&
           (reinterpret_cast<uintptr_t>(X) % 16) == 0;
}

int plain_wave_quantize(const void* X, int dtype, int64_t rows, int d, int64_t ld, int bits, float clip,
                        uint32_t* codes, float* scales, hipStream_t s) {
    const PlainArgs a{static_cast<const uint16_t*>(X), rows, d, ld, codes, scales, (double)clip, dtype == RQ_F16};
    const int t = (d + 511) / 512;
    if (t <= 1) return launch_plain<1>(a, bits, s);
    if (t <= 2) return launch_plain<2>(a, bits, s);
    if (t <= 4) return launch_plain<4>(a, bits, s);
    if (t <= 8) return launch_plain<8>(a, bits, s);
    if (t <= 16) return launch_plain<16>(a, bits, s);
    if (t <= 24) return launch_plain<24>(a, bits, s);
    return launch_plain<40>(a, bits, s);
}

bool wave_asym_supports(const rq_hadamard* h, const RowArgs& a) {
    return wave_supports(h, a) && a.log2m == 7;
}

int wave_rotate_quantize_asym(const rq_hadamard* h, const RowArgs& a, float clip, uint32_t* codes,
                              float* scales, float* mins, hipStream_t s) {
    const double lvl = (double)((1 << a.bits) - 1);
    const double rn = std::sqrt((double)a.n);
    WaveArgs w{static_cast<const uint16_t*>(a.X), a.rows, a.d, a.ld,
               static_cast<const u32x4*>(h->d_tiles), codes, scales,
               lvl / (double)clip, (double)clip / (rn * lvl), mins, (double)clip, (double)clip / rn};
    if (a.dtype == RQ_F16) {
        w.f16 = true;
        w.tiles = static_cast<const u32x4*>(h->d_tiles_f16);
    }
    return launch_short_asym(h, w, a.bits, s);
}

}  // namespace rq
