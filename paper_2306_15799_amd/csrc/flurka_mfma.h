// Building blocks for the bf16 MFMA kernels (gfx950).
#pragma once

#include "flurka_internal.h"

namespace flurka {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

// v_mfma_f32_32x32x16_bf16, one wavefront: D(32x32) += A(32x16) B(16x32).
// Operand layout, lane l (verified on hardware):
//   A: row l%32, reduction slots 8*(l/32) .. +7        (8 bf16, 16 bytes)
//   B: column l%32, reduction slots 8*(l/32) .. +7
//   D: column l%32, element g (0..15) is row 8*(g/4) + 4*(l/32) + g%4
__device__ __forceinline__ floatx16 mfma32(const uint4& a, const uint4& b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ floatx16 zero16() {
    floatx16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;

// two floats -> packed bf16 pair (low half = a), round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    const floatx2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Split-precision operands: x = hi + lo (+ more) with every term a bf16, two values at a time on the
// packed hardware conversion (round to nearest even).  pair_lo/pair_hi widen the halves of a packed pair.
__device__ __forceinline__ float pair_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float pair_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
__device__ __forceinline__ void split2_pair(float x0, float x1, uint32_t& hi, uint32_t& lo) {
    hi = pack_bf16(x0, x1);
    lo = pack_bf16(x0 - pair_lo(hi), x1 - pair_hi(hi));
}
__device__ __forceinline__ void split3_pair(float x0, float x1, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    hi = pack_bf16(x0, x1);
    const float r0 = x0 - pair_lo(hi), r1 = x1 - pair_hi(hi);
    mid = pack_bf16(r0, r1);
    lo = pack_bf16(r0 - pair_lo(mid), r1 - pair_hi(mid));
}

// 2^x on the transcendental unit, no denormal fix-up (inputs here are <= 0 and results that
// underflow are meant to be 0)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint4 ld16(const void* p) { return *(const uint4*)p; }

// Combine the values that lanes l and l ^ 32 hold (the two halves of a wavefront carry the two
// halves of an MFMA reduction).  v_permlane32_swap exchanges the upper half of one register with the
// lower half of another, so two copies of x become {lo, lo} and {hi, hi}: no LDS round trip.
__device__ __forceinline__ float half_max(float x) {
    const unsigned xi = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    const unsigned xi = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// A 32x32 accumulator gives lane l rows 8q + 4*(l/32) + {0..3} of its column: lanes l and l ^ 32
// hold the two 8-byte halves of every 8-row group.  Given the packed halves of groups 2i (`even`)
// and 2i + 1 (`odd`), one v_permlane32_swap per dword leaves each lane with ONE complete group --
// group 2i + (l/32) -- so results can be stored 16 bytes at a time.
__device__ __forceinline__ uint4 join_halves(uint2 even, uint2 odd) {
    const auto x = __builtin_amdgcn_permlane32_swap(even.x, odd.x, false, false);
    const auto y = __builtin_amdgcn_permlane32_swap(even.y, odd.y, false, false);
    return make_uint4(x[0], y[0], x[1], y[1]);
}

// Value that lane G of this lane's row of 16 lanes holds (DPP row_newbcast, no LDS traffic).  With
// one register per 32-feature tile loaded so that lane 16*r + n holds the entry for accumulator
// element n of half r/2, bcast16<g>(reg) is the entry that belongs to accumulator element g.
template <int G>
__device__ __forceinline__ float bcast16(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + G, 0xf, 0xf, false));
}
// lane's position in a per-tile vector stored in accumulator order (slot 16*half + g)
__device__ __forceinline__ int acc_order_slot(int lane) { return 16 * (lane >> 5) + (lane & 15); }

constexpr float FLURKA_LOG2E = 1.4426950408889634f;
// The running row maximum is only raised when a tile exceeds it by more than this (natural log
// units): weights may then be as large as exp(40) = 2.4e17 instead of 1 and a row's sums reach 1e20,
// which costs nothing in fp32 or bf16 range (both end near 3e38), and the rescaling of the accumulators
// stays out of almost every tile.  (The per-feature shifts c' spread over tens of units, so with a small
// margin the maximum keeps creeping up from tile to tile.)
constexpr float FLURKA_LAZY_MAX = 40.0f;

// Forward pass over all feature tiles for the 32 query rows of one wavefront (lane = query):
//   u^T = [omega | c'] [q | 1]^T -> running max mu -> P'^T = exp -> N^T += S'^T P'^T (P'^T goes from the
//   accumulator registers straight into the B operand), den += sum of the bf16 P'.
// The key side hands over S'_j = S_j / z_j and c'_j = c_j + ln z_j, so that P'_ij = P_ij z_j: the
// denominator is a plain sum, and the shift enters the first contraction as one more reduction step
// (three bf16 terms of c' against ones): no per-feature vector is touched on the VALU, which is the
// unit this loop is bound by.
// An in-order wavefront overlaps its matrix and vector pipes only if the two kinds of instruction
// alternate in program order, so the loop is software-pipelined by hand: iteration ft runs the exp
// work of tile ft, and between those VALU groups issues the (dependent) MFMAs of u^T for tile ft + 1
// and the MFMAs of N^T for tile ft; the maximum of tile ft + 1 is taken in the shadow of the last
// N^T MFMAs.  sched_barrier(0) after each group pins the order.  The only branch is the (rare, see
// FLURKA_LAZY_MAX) rescaling between iterations.
// lw: [omega | c' terms | 0] rows [feature][D + 16] (pitch w_pitch), ls: S'^T [t][feature slot] (pitch
// s_pitch); both in LDS.
// `last_hook()` runs at the start of the last iteration, which no longer needs qf: a caller that
// streams over query tiles issues the loads of its next tile there (it may overwrite qf).
template <int N> struct IterTag { static constexpr int value = N; };

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 flurka_bf16x2;
// acc + lo(p) + hi(p) for a packed pair of bf16
__device__ __forceinline__ float add_bf16_pair(uint32_t p, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(flurka_bf16x2, p),
                                           __builtin_bit_cast(flurka_bf16x2, 0x3f803f80u), acc, false);
}

template <int D, int QT, class LastHook>
__device__ __forceinline__ void forward_feature_pass(const unsigned char* lw, int w_pitch, const unsigned char* ls,
                                                     int s_pitch, int FT, int l32, int half,
                                                     uint4 (&qf)[QT][D / 16], floatx16 (&accN)[QT][D / 32],
                                                     float (&den)[QT], float (&mu)[QT], LastHook&& last_hook) {
    constexpr int KS = D / 16, TT = D / 32;
    constexpr int EPC = 16 / KS;                 // accumulator elements handled per group
    const unsigned char* wrow = lw + l32 * w_pitch + 16 * half;        // + 32*ft rows, + 32*s
    const unsigned char* srow = ls + l32 * s_pitch + 16 * half;        // + 32*t rows, + 64*ft (+32)
    // B operand of the extra reduction step: ones against the three terms of c' (slots 0..2)
    const uint4 qone = half == 0 ? make_uint4(0x3f803f80u, 0x00003f80u, 0u, 0u) : make_uint4(0u, 0u, 0u, 0u);

    auto tile_max = [&](const floatx16& u) -> float {
        float tmax = fmaxf(fmaxf(u[0], u[1]), u[2]);
#pragma unroll
        for (int g = 3; g < 15; g += 2) tmax = fmaxf(fmaxf(tmax, u[g]), u[g + 1]);
        return half_max(fmaxf(tmax, u[15]));
    };
    auto maybe_rescale = [&](int i, float tmax) {
        if (tmax > mu[i] + FLURKA_LAZY_MAX) {
            const float sc = fast_exp2((mu[i] - tmax) * FLURKA_LOG2E);
            mu[i] = tmax;
            den[i] *= sc;
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
                for (int g = 0; g < 16; ++g) accN[i][t][g] *= sc;
        }
    };

    // prologue: tile 0
    floatx16 u[QT];
    {
#pragma unroll
        for (int i = 0; i < QT; ++i) u[i] = zero16();
#pragma unroll
        for (int s = 0; s <= KS; ++s) {
            const uint4 wa = *(const uint4*)(wrow + 32 * s);
#pragma unroll
            for (int i = 0; i < QT; ++i) u[i] = mfma32(wa, s < KS ? qf[i][s] : qone, u[i]);
        }
        // the first tile's maximum simply becomes the running maximum: nothing has been accumulated
        // yet, so there is nothing to rescale
#pragma unroll
        for (int i = 0; i < QT; ++i) mu[i] = tile_max(u[i]);
    }

    auto iteration = [&](int ft, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value != 0;
        const int nft = LAST ? ft : ft + 1;
        float nshift[QT];
        floatx16 un[QT];
        if constexpr (LAST) last_hook();
#pragma unroll
        for (int i = 0; i < QT; ++i) nshift[i] = -mu[i] * FLURKA_LOG2E;
        uint4 wa[KS + 1], sa[2 * TT];
        if constexpr (!LAST) {
#pragma unroll
            for (int s = 0; s <= KS; ++s) wa[s] = *(const uint4*)(wrow + (32 * nft) * w_pitch + 32 * s);
        }
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            sa[2 * t] = *(const uint4*)(srow + (32 * t) * s_pitch + 64 * ft);
            sa[2 * t + 1] = *(const uint4*)(srow + (32 * t) * s_pitch + 64 * ft + 32);
        }
        if constexpr (!LAST) {
            // the shift step opens the chain of the next tile's u^T
#pragma unroll
            for (int i = 0; i < QT; ++i) un[i] = mfma32(wa[KS], qone, zero16());
        }
        __builtin_amdgcn_sched_barrier(0);
        uint32_t pk[QT][8];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            // dependent MFMAs of the next tile's u^T (one per query tile) ...
            if constexpr (!LAST) {
#pragma unroll
                for (int i = 0; i < QT; ++i) un[i] = mfma32(wa[s], qf[i][s], un[i]);
            }
            // ... over the exp work of EPC elements of this tile
#pragma unroll
            for (int i = 0; i < QT; ++i) {
                float p[EPC];
#pragma unroll
                for (int e = 0; e < EPC; ++e) p[e] = fast_exp2(fmaf(u[i][s * EPC + e], FLURKA_LOG2E, nshift[i]));
#pragma unroll
                for (int e = 0; e < EPC; e += 2) {
                    pk[i][(s * EPC + e) / 2] = pack_bf16(p[e], p[e + 1]);
                    den[i] = add_bf16_pair(pk[i][(s * EPC + e) / 2], den[i]);
                }
            }
            // second half of the groups: N^T MFMAs with the first half of P^T (elements 0..7)
            if (s >= KS / 2) {
                constexpr int per = (TT + KS / 2 - 1) / (KS / 2);
#pragma unroll
                for (int j = 0; j < per; ++j) {
                    const int t = (s - KS / 2) * per + j;
                    if (t < TT) {
#pragma unroll
                        for (int i = 0; i < QT; ++i)
                            accN[i][t] = mfma32(sa[2 * t], make_uint4(pk[i][0], pk[i][1], pk[i][2], pk[i][3]), accN[i][t]);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // N^T MFMAs with the second half of P^T, over the maximum of the next tile
        float tmax[QT];
        if constexpr (!LAST) {
#pragma unroll
            for (int i = 0; i < QT; ++i) tmax[i] = fmaxf(fmaxf(un[i][0], un[i][1]), un[i][2]);
        }
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            constexpr int per = (12 + TT - 1) / TT;          // elements 3..14 spread over the TT groups
#pragma unroll
            for (int i = 0; i < QT; ++i) {
                accN[i][t] = mfma32(sa[2 * t + 1], make_uint4(pk[i][4], pk[i][5], pk[i][6], pk[i][7]), accN[i][t]);
                if constexpr (!LAST) {
#pragma unroll
                    for (int g = 3 + t * per; g < 3 + (t + 1) * per && g < 15; ++g) tmax[i] = fmaxf(tmax[i], un[i][g]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (!LAST) {
#pragma unroll
            for (int i = 0; i < QT; ++i) {
                tmax[i] = half_max(fmaxf(tmax[i], un[i][15]));
                maybe_rescale(i, tmax[i]);
                u[i] = un[i];
            }
        }
    };
    for (int ft = 0; ft + 1 < FT; ++ft) iteration(ft, IterTag<0>{});
    iteration(FT - 1, IterTag<1>{});
}

}  // namespace flurka
