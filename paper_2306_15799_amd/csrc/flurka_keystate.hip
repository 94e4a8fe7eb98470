// Key-side state of FLuRKA attention on MFMA (gfx950):  S = PhiK^T V',  z = PhiK^T 1,  c.
//
// PhiK_rj = exp(e_rj - c_j),  e_rj = omega_j . k'_r - |k'_r|^2 / 2  (positive random features, Sec. 2
// "Kernel Methods"), or PhiK = elu(K') + 1.  exp() turns an absolute error of e into a relative error
// of the attention weights, and |e| reaches several hundred for long sequences, so e is formed to
// fp32 accuracy: K' (fp32) is split into three bf16 terms whose products with the bf16 omega are
// exact in the fp32 accumulator.  PhiK and V' enter the second contraction as two-term bf16 splits.
//
// Two kernels:
//   proj_finish   sums the projection's split-n partials into K', V' (fp32, ctx) and writes the
//                 operand images: K' as bf16 hi/mid/lo rows, V' as bf16 hi/lo with two consecutive
//                 keys per dword, and |k'|^2 / 2 per key
//   key_state     one workgroup per (head, 32 features), one wavefront per key range: first
//                 contraction on MFMA, column maximum, exp, second contraction on MFMA with PhiK taken
//                 from the accumulator registers as the A operand; the ranges' partial S, z, c meet in
//                 LDS, are joined there (log-sum-exp style) and leave as S, z, c (fp32, ctx) and as the
//                 bf16 images the query-stream kernel loads into LDS
#include "flurka_fast.h"
#include "flurka_gemm.h"

namespace flurka {

#define FLURKA_CHECK_LAUNCH()                                   \
    do {                                                        \
        if (hipGetLastError() != hipSuccess) return FLURKA_ERR_LAUNCH; \
    } while (0)

static inline dim3 grid1d(long total, int block) { return dim3((unsigned)((total + block - 1) / block)); }

// x = hi + mid + lo with each term a bf16 (24 mantissa bits in total)
__device__ __forceinline__ void split3(float x, uint16_t& hi, uint16_t& mid, uint16_t& lo) {
    hi = f32_to_bf16(x);
    const float r1 = x - bf16_to_f32(hi);
    mid = f32_to_bf16(r1);
    lo = f32_to_bf16(r1 - bf16_to_f32(mid));
}

// ---------------------------------------------------------------------------
// proj_finish: one wavefront per (head, four consecutive keys 4g .. 4g+3); lane = coordinate t (and
// t + 64 for d = 128).  The four keys are the four floats of one 16-byte element of the projection's
// tile-ordered partial results, and consecutive t are consecutive elements: coalesced float4 loads.
// ---------------------------------------------------------------------------
struct FinishArgs {
    const float* part;      // tile-ordered split partials of the projection (see flurka_gemm.h)
    float* ctx;             // K' at ctx + Kp_off, V' at ctx + Vp_off
    long Kp_off, Vp_off;
    uint16_t* Kimg;         // 3 x (BH, kpad * d) bf16: hi, mid, lo, in key_state's operand order (nullptr for elu1)
    uint32_t* Vimg;         // 2 x (BH, kpad/2, d) dwords: hi, lo; low half = even key (nullptr: K', V' only)
    float* nrm;             // (BH, kpad): |k'|^2/2, +inf for the padding keys (nullptr for elu1)
    int splits, tilesM, tilesN, k, kpad, d, BH;
};

__global__ __launch_bounds__(256) void proj_finish_kernel(FinishArgs a) {
    const int lane = threadIdx.x & 63;
    const long wid = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int groups_per_head = a.kpad / 4;
    if (wid >= (long)a.BH * groups_per_head) return;
    const int bh = (int)(wid / groups_per_head);
    const int r0 = 4 * (int)(wid % groups_per_head);           // keys r0 .. r0 + 3
    const int hpt = GBN / a.d;                                  // heads per column tile
    const int tn = bh / hpt, tm = r0 / GBM;
    const long img_plane = (long)a.BH * a.kpad * a.d;          // elements per K image plane
    const long vimg_plane = (long)a.BH * (a.kpad / 2) * a.d;
    float sq[4] = {0.f, 0.f, 0.f, 0.f};
    for (int t = lane; t < a.d; t += 64) {
        const int eo = partial_elem_offset(r0 % GBM, (bh % hpt) * a.d + t);
        float4 ks = {0.f, 0.f, 0.f, 0.f}, vs = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < a.splits; ++s) {
            const float4 x = *(const float4*)(a.part + partial_tile_index(0, s, tn, tm, a.splits, a.tilesN, a.tilesM) * G_TILE_ELEMS + eo);
            const float4 y = *(const float4*)(a.part + partial_tile_index(1, s, tn, tm, a.splits, a.tilesN, a.tilesM) * G_TILE_ELEMS + eo);
            ks.x += x.x; ks.y += x.y; ks.z += x.z; ks.w += x.w;
            vs.x += y.x; vs.y += y.y; vs.z += y.z; vs.w += y.w;
        }
        float kv[4] = {ks.x, ks.y, ks.z, ks.w}, vv[4] = {vs.x, vs.y, vs.z, vs.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int r = r0 + e;
            if (r < a.k) {
                const long off = ((long)bh * a.k + r) * a.d + t;
                a.ctx[a.Kp_off + off] = kv[e];
                a.ctx[a.Vp_off + off] = vv[e];
            } else {
                kv[e] = 0.f; vv[e] = 0.f;                      // rows of a tile past k hold nothing useful
            }
            sq[e] = fmaf(kv[e], kv[e], sq[e]);
            if (a.Kimg) {
                uint16_t hi, mid, lo;
                split3(kv[e], hi, mid, lo);
                // operand order of key_state: [32-key tile][16-coordinate step][8-coordinate half][key][8],
                // so that a wavefront's fragment load is 1 KiB of consecutive bytes
                const long io = (long)bh * a.kpad * a.d +
                                ((((long)(r >> 5) * (a.d / 16) + (t >> 4)) * 2 + ((t >> 3) & 1)) * 32 + (r & 31)) * 8 + (t & 7);
                a.Kimg[io] = hi;
                a.Kimg[img_plane + io] = mid;
                a.Kimg[2 * img_plane + io] = lo;
            }
        }
#pragma unroll
        for (int pr = 0; pr < 2 && a.Vimg; ++pr) {
            uint32_t hp, lp;
            split2_pair(vv[2 * pr], vv[2 * pr + 1], hp, lp);
            const long vo = ((long)bh * (a.kpad / 2) + r0 / 2 + pr) * a.d + t;
            a.Vimg[vo] = hp;
            a.Vimg[vimg_plane + vo] = lp;
        }
    }
    if (a.nrm) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float tot = wave_sum(sq[e]);
            const int r = r0 + e;
            if (lane == 0) a.nrm[(long)bh * a.kpad + r] = r < a.k ? 0.5f * tot : INFINITY;
        }
    }
}

// ---------------------------------------------------------------------------
// key_state: one wavefront per (head, feature tile, key range)
// ---------------------------------------------------------------------------
struct KeyStateArgs {
    const uint16_t* Kimg;   // performer
    const float* Kp;        // elu1: K' fp32 (BH, k, d)
    const uint16_t* Kb;     // elu1, EXACT: the keys themselves, bf16 (BH, k, d)
    const uint32_t* Vimg;
    const float* nrm;
    const uint16_t* omega;
    float* S; float* z; float* c;            // ctx
    uint16_t* St; float* zp; uint16_t* cw;   // images for the query stream (see the merge step below)
    long omega_head_stride;
    int BH, H, k, kpad, mf, mfp, FT, KR, tiles_per_range;   // mf features (ctx strides), mfp = mf rounded up to whole tiles (image strides)
};

// LDS of a workgroup: per key range the partial S tile (32 features x d, rows padded), z and c; then
// the merge step's weights, 1/z and one 32 x 32 transposition tile.
template <int D>
struct KeyStateLds {
    static constexpr int s_pitch = D + 4;                                   // floats
    static __host__ __device__ int range_floats() { return 32 * s_pitch + 64; }
    static __host__ __device__ int total(int KR) { return (KR * range_floats() + KR * 32 + 32 + 32 * 33) * 4; }
};

// key tiles of a range that stay in registers (head size 128 keeps fewer, and does without the
// one-tile-ahead request of V' below: its eight wavefronts per workgroup share 256 registers each)
template <int D> struct KeyStateKeep { static constexpr int value = D <= 64 ? 4 : 2; };

// most wavefronts (key ranges) per workgroup: what the kernel's register need leaves room for
template <int D> struct KeyStateMaxWaves { static constexpr int value = 8; };

// EXACT: the keys and values are bf16 numbers to begin with (kernel attention without a sequence
// projection): one term of K and one of V carry everything, the other operand terms are skipped.
template <int D, bool ELU, bool EXACT>
__global__ __launch_bounds__(KeyStateMaxWaves<D>::value * 64) void key_state_kernel(KeyStateArgs a) {
    constexpr int KS = D / 16, TT = D / 32;
    extern __shared__ __attribute__((aligned(16))) float ks_lds[];
    using L = KeyStateLds<D>;
    const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
    const int kr = threadIdx.x >> 6;                       // this wavefront's key range
    // Workgroup ids go round the 8 XCDs; the FT workgroups of one head all read that head's K' and V'
    // images, so they take ids that are equal mod 8 and share one L2.
    const int slot = (int)(blockIdx.x >> 3);
    const int ft = slot % a.FT;
    const int bh = (slot / a.FT) * 8 + (int)(blockIdx.x & 7);
    if (bh >= a.BH) return;                                // head count rounded up to whole groups of 8
    const int KT = a.kpad / 32;
    const int kt0 = kr * a.tiles_per_range;
    int kt1 = kt0 + a.tiles_per_range;
    if (kt1 > KT) kt1 = KT;
    const long plane = (long)a.BH * a.kpad * D;
    const long vplane = (long)a.BH * (a.kpad / 2) * D;
    const uint32_t* vimg = a.Vimg + (long)bh * (a.kpad / 2) * D;

    // B operand of the first contraction: omega rows of this feature tile
    uint4 wf[KS];
    if (!ELU) {
        // features past mf (a ragged last tile) take the last real row; their results are replaced below
        const int fr = 32 * ft + l32 < a.mf ? 32 * ft + l32 : a.mf - 1;
        const uint16_t* og = a.omega + (long)(bh % a.H) * a.omega_head_stride + (long)fr * D + 8 * half;
#pragma unroll
        for (int s = 0; s < KS; ++s) wf[s] = ld16(og + 16 * s);
    }

    // exponents (performer) or features (elu1) of one 32-key tile: lane = feature 32*ft + l32,
    // element g = key 32*kt + 8*(g/4) + 4*half + g%4
    auto tile_values = [&](int kt) -> floatx16 {
        floatx16 e = zero16();
        if (!ELU) {
            const uint16_t* kg = a.Kimg + (long)bh * a.kpad * D + ((long)kt * KS * 64 + lane) * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                e = mfma32(ld16(kg + 512 * s), wf[s], e);
                if constexpr (!EXACT) {
                    e = mfma32(ld16(kg + plane + 512 * s), wf[s], e);
                    e = mfma32(ld16(kg + 2 * plane + 512 * s), wf[s], e);
                }
            }
            const float* ng = a.nrm + (long)bh * a.kpad + 32 * kt + 4 * half;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 nq = *(const float4*)(ng + 8 * q);
                e[4 * q] -= nq.x; e[4 * q + 1] -= nq.y; e[4 * q + 2] -= nq.z; e[4 * q + 3] -= nq.w;
            }
        } else {
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const int r = 32 * kt + 8 * (g >> 2) + 4 * half + (g & 3);
                float v = 0.f;                                    // padding keys contribute nothing
                if (r < a.k) {
                    const long idx = ((long)bh * a.k + r) * D + 32 * ft + l32;
                    const float x = EXACT ? bf16_to_f32(a.Kb[idx]) : a.Kp[idx];
                    v = x > 0.f ? x + 1.f : __expf(x);
                }
                e[g] = v;
            }
        }
        return e;
    };

    // B operands of the second contraction for one key tile: V' columns 32*tt + l32, key pairs in the
    // order in which the accumulator hands PhiK^T on.  They are requested a tile ahead, so that the trip
    // to memory runs under the exponentials of the tile before (one wavefront per SIMD: nobody else
    // would hide it).
    struct VFrag { uint4 h[2][TT], l[2][TT]; };
    auto load_v = [&](int kt, VFrag& f) {
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
            const uint32_t* vb = vimg + (long)(16 * kt + 8 * sp + 2 * half) * D + l32;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                f.h[sp][tt].x = vb[32 * tt];
                f.h[sp][tt].y = vb[32 * tt + D];
                f.h[sp][tt].z = vb[32 * tt + 4 * D];
                f.h[sp][tt].w = vb[32 * tt + 5 * D];
                if constexpr (!EXACT) {
                    f.l[sp][tt].x = vb[vplane + 32 * tt];
                    f.l[sp][tt].y = vb[vplane + 32 * tt + D];
                    f.l[sp][tt].z = vb[vplane + 32 * tt + 4 * D];
                    f.l[sp][tt].w = vb[vplane + 32 * tt + 5 * D];
                }
            }
        }
    };
    // Up to KS_MT tiles per range (what the plan aims for) are evaluated once, all their loads in flight
    // together, and kept in registers between the maximum and the accumulation; longer ranges are
    // evaluated twice.
    const int nt = kt1 - kt0;
    constexpr int KS_MT = KeyStateKeep<D>::value;
    constexpr bool V_AHEAD = D <= 64;
    const bool keep = nt <= KS_MT;
    floatx16 ev[KS_MT];
    if (keep) {
#pragma unroll
        for (int i = 0; i < KS_MT; ++i)
            if (i < nt) ev[i] = tile_values(kt0 + i);
    }
    VFrag vcur, vnext;
    load_v(kt0, vcur);
    float c = 0.f;
    if (!ELU) {
        c = -INFINITY;
        if (keep) {
#pragma unroll
            for (int i = 0; i < KS_MT; ++i)
                if (i < nt) {
#pragma unroll
                    for (int g = 0; g < 16; ++g) c = fmaxf(c, ev[i][g]);
                }
        } else {
            for (int kt = kt0; kt < kt1; ++kt) {
                const floatx16 e = tile_values(kt);
#pragma unroll
                for (int g = 0; g < 16; ++g) c = fmaxf(c, e[g]);
            }
        }
        c = half_max(c);
    }

    floatx16 accS[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) accS[t] = zero16();
    float zsum = 0.f;
    constexpr float LOG2E = 1.4426950408889634f;
    auto accumulate = [&](const floatx16& e, const VFrag& f) {
        uint32_t hi[8], lo[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float p0 = e[2 * q], p1 = e[2 * q + 1];
            if (!ELU) {
                p0 = fast_exp2((p0 - c) * LOG2E);
                p1 = fast_exp2((p1 - c) * LOG2E);
            }
            zsum += p0 + p1;
            split2_pair(p0, p1, hi[q], lo[q]);
        }
        // PhiK^T tile as A operand: row = this lane's feature, reduction slots = keys in accumulator order
        const uint4 ah[2] = {{hi[0], hi[1], hi[2], hi[3]}, {hi[4], hi[5], hi[6], hi[7]}};
        const uint4 al[2] = {{lo[0], lo[1], lo[2], lo[3]}, {lo[4], lo[5], lo[6], lo[7]}};
#pragma unroll
        for (int sp = 0; sp < 2; ++sp)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                accS[tt] = mfma32(ah[sp], f.h[sp][tt], accS[tt]);
                accS[tt] = mfma32(al[sp], f.h[sp][tt], accS[tt]);
                if constexpr (!EXACT) accS[tt] = mfma32(ah[sp], f.l[sp][tt], accS[tt]);
            }
    };
    {
        if (keep) {
#pragma unroll
            for (int i = 0; i < KS_MT; ++i)
                if (i < nt) {
                    if constexpr (V_AHEAD) {
                        if (i + 1 < nt) load_v(kt0 + i + 1, vnext);
                        accumulate(ev[i], vcur);
                        if (i + 1 < nt) vcur = vnext;
                    } else {
                        if (i > 0) load_v(kt0 + i, vcur);
                        accumulate(ev[i], vcur);
                    }
                }
        } else {
            for (int kt = kt0; kt < kt1; ++kt) {
                if constexpr (V_AHEAD) {
                    if (kt + 1 < kt1) load_v(kt + 1, vnext);
                    accumulate(tile_values(kt), vcur);
                    if (kt + 1 < kt1) vcur = vnext;
                } else {
                    if (kt > kt0) load_v(kt, vcur);
                    accumulate(tile_values(kt), vcur);
                }
            }
        }
    }
    zsum = half_sum(zsum);

    // this range's partial results into LDS: S tile [feature][t], then z[32], c[32]
    float* const mine = ks_lds + kr * L::range_floats();
    if (half == 0) {
        mine[32 * L::s_pitch + l32] = zsum;
        mine[32 * L::s_pitch + 32 + l32] = c;
    }
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            const int f = 8 * (g >> 2) + 4 * half + (g & 3);
            mine[f * L::s_pitch + 32 * tt + l32] = accS[tt][g];
        }
    __syncthreads();

    // Merge of the key ranges, by the whole workgroup:
    //   c_j = max_r c_jr,  S_j = sum_r exp(c_jr - c_j) S_jr,  z_j likewise
    //   St (d x mf) bf16: St[t][slot] = S[feature(slot)][t];  zp: z in accumulator order of a tile
    // For the random-feature map the query stream works with p'_ij = p_ij z_j, so that its denominator
    // is the plain sum of p': St holds S_j / z_j, and cw the exponent shift c_j + ln z_j as three bf16
    // terms (it enters the query kernel's first contraction as extra reduction slots against ones).
    // The slot -> feature order inside each group of 16 is the order in which the first MFMA of the
    // query-stream kernel hands P^T on as the B operand of the second:
    //   slot 16*q + 8*h + e  <->  feature 16*q + 8*(e/4) + 4*h + e%4          (natural order for elu1)
    const int KR = a.KR, tid = threadIdx.x, nthreads = blockDim.x;
    float* const wgt = ks_lds + KR * L::range_floats();      // [range][feature]
    float* const zinv = wgt + KR * 32;
    float* const tile = zinv + 32;                           // [32][33]
    if (tid < 32) {
        const int f = 32 * ft + tid;
        float cm = -INFINITY;
        for (int r = 0; r < KR; ++r) cm = fmaxf(cm, ks_lds[r * L::range_floats() + 32 * L::s_pitch + 32 + tid]);
        float zs = 0.f;
        for (int r = 0; r < KR; ++r) {
            const float* pr = ks_lds + r * L::range_floats() + 32 * L::s_pitch;
            const float wr = ELU ? 1.f : expf(pr[32 + tid] - cm);
            wgt[r * 32 + tid] = wr;
            zs = fmaf(wr, pr[tid], zs);
        }
        const bool real = f < a.mf;              // a feature of the padding: weight exp(-1e30) = 0 in the query stream
        if (real) {
            a.z[(long)bh * a.mf + f] = zs;
            a.c[(long)bh * a.mf + f] = cm;
        }
        // accumulator order of a 32-feature tile: position 16*h + g <-> feature 8*(g/4) + 4*h + g%4
        int pos = tid;
        if (!ELU) {
            const int q = tid >> 3, h = (tid >> 2) & 1, e = tid & 3;
            pos = 16 * h + 4 * q + e;
        }
        a.zp[(long)bh * a.mfp + 32 * ft + pos] = zs;
        if (!ELU) {
            uint16_t hi, mid, lo;
            split3(real ? cm + logf(zs) : -1e30f, hi, mid, lo);
            uint2 pk;
            pk.x = (uint32_t)hi | ((uint32_t)mid << 16);
            pk.y = (uint32_t)lo;
            *(uint2*)(a.cw + ((long)bh * a.mfp + f) * 4) = pk;
        }
        zinv[tid] = ELU ? 1.f : (real ? 1.f / zs : 0.f);
    }
    __syncthreads();
    for (int t0 = 0; t0 < D; t0 += 32) {
        for (int i = tid; i < 32 * 32; i += nthreads) {
            const int fl = i / 32, t = t0 + i % 32;
            float sv = 0.f;
            for (int r = 0; r < KR; ++r)
                sv = fmaf(wgt[r * 32 + fl], ks_lds[r * L::range_floats() + fl * L::s_pitch + t], sv);
            if (32 * ft + fl < a.mf) a.S[((long)bh * a.mf + 32 * ft + fl) * D + t] = sv;
            tile[fl * 33 + i % 32] = sv;
        }
        __syncthreads();
        for (int i = tid; i < 32 * 32; i += nthreads) {
            const int tl = i / 32, sl = i % 32;
            int fl = sl;
            if (!ELU) {
                const int e = sl & 7, h = (sl >> 3) & 1;
                fl = (sl & 16) + 8 * (e >> 2) + 4 * h + (e & 3);
            }
            a.St[((long)bh * D + t0 + tl) * a.mfp + 32 * ft + sl] = f32_to_bf16(tile[fl * 33 + tl] * zinv[fl]);
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
KeyStatePlan key_state_plan(const Problem& p) {
    KeyStatePlan q;
    q.kpad = (p.k + 31) / 32 * 32;
    q.FT = p.mfp / 32;
    const int KT = q.kpad / 32;
    // Key ranges = wavefronts of a workgroup: about two key tiles per wavefront (measured best at the
    // benchmark shapes: fewer wavefronts leave the latency of the operand loads exposed, more of them
    // make the merge longer), at most KeyStateMaxWaves (the ranges' partial tiles meet in LDS).  Ranges
    // of more than KeyStateKeep tiles are evaluated twice (maximum, then accumulation).
    const int max_kr = p.d <= 64 ? KeyStateMaxWaves<64>::value : KeyStateMaxWaves<128>::value;
    const int want = (KT + 1) / 2;
    int KR = 1;
    while (KR < want && KR < max_kr) KR *= 2;
    while (KR > KT && KR > 1) KR /= 2;
    q.tiles_per_range = (KT + KR - 1) / KR;
    q.KR = (KT + q.tiles_per_range - 1) / q.tiles_per_range;
    return q;
}

template <int D, bool ELU, bool EXACT>
static flurka_status launch_key_state_impl(const Problem& p, const KeyStateArgs& ka, hipStream_t s) {
    auto kern = key_state_kernel<D, ELU, EXACT>;
    const int ldsb = KeyStateLds<D>::total(ka.KR);
    KernelFacts facts;
    if (!kernel_facts((const void*)kern, ka.KR * 64, ldsb, &facts)) return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)((p.BH + 7) / 8 * 8 * ka.FT)), dim3(ka.KR * 64), ldsb, s, ka);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

template <int D>
static flurka_status launch_key_state(const Problem& p, const KeyStateArgs& ka, bool exact, hipStream_t s) {
    if (exact) return p.elu ? launch_key_state_impl<D, true, true>(p, ka, s) : launch_key_state_impl<D, false, true>(p, ka, s);
    return p.elu ? launch_key_state_impl<D, true, false>(p, ka, s) : launch_key_state_impl<D, false, false>(p, ka, s);
}

flurka_status fast_proj_finish(const Problem& p, float* ctx, const float* partials, int tilesM, int tilesN,
                               int splits, bool images, const KeyStateBuffers& b, hipStream_t s) {
    const CtxLayout L = ctx_layout(p);
    const KeyStatePlan q = key_state_plan(p);
    StageScope sc(s, STAGE_K_PROJ_FINISH);
    FinishArgs fa{};
    fa.part = partials; fa.ctx = ctx; fa.tilesM = tilesM; fa.tilesN = tilesN;
    fa.Kp_off = (long)L.Kp; fa.Vp_off = (long)L.Vp;
    fa.Kimg = (p.elu || !images) ? nullptr : b.Kimg; fa.Vimg = images ? b.Vimg : nullptr;
    fa.nrm = (p.elu || !images) ? nullptr : b.nrm;
    fa.splits = splits; fa.k = p.k; fa.kpad = q.kpad; fa.d = p.d; fa.BH = p.BH;
    const long waves = (long)p.BH * (q.kpad / 4);
    hipLaunchKernelGGL(proj_finish_kernel, grid1d(waves, 4), dim3(256), 0, s, fa);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

flurka_status fast_key_state(const Problem& p, const void* omega, float* ctx, const float* partials,
                             int tilesM, int tilesN, int splits, const KeyStateBuffers& b, hipStream_t s) {
    const CtxLayout L = ctx_layout(p);
    const KeyStatePlan q = key_state_plan(p);
    {
        const flurka_status st = fast_proj_finish(p, ctx, partials, tilesM, tilesN, splits, true, b, s);
        if (st != FLURKA_OK) return st;
    }
    {
        StageScope sc(s, STAGE_K_KEY_STATE);
        KeyStateArgs ka{};
        ka.Kimg = b.Kimg; ka.Kp = ctx + L.Kp; ka.Vimg = b.Vimg; ka.nrm = b.nrm;
        ka.omega = (const uint16_t*)omega;
        ka.S = ctx + L.S; ka.z = ctx + L.z; ka.c = ctx + L.c;
        ka.St = b.St; ka.zp = b.zp; ka.cw = b.cw;
        ka.omega_head_stride = p.omega_per_head ? (long)p.m * p.d : 0;
        ka.BH = p.BH; ka.H = p.H; ka.k = p.k; ka.kpad = q.kpad; ka.mf = p.mf; ka.mfp = p.mfp;
        ka.FT = q.FT; ka.KR = q.KR; ka.tiles_per_range = q.tiles_per_range;
        flurka_status st = p.d == 64 ? launch_key_state<64>(p, ka, false, s) : launch_key_state<128>(p, ka, false, s);
        if (st != FLURKA_OK) return st;
    }
    return FLURKA_OK;
}

// ---------------------------------------------------------------------------
// Kernel attention without a sequence projection (K' = K, V' = V): the keys and values are the caller's
// bf16 tensors.  identity_pack writes what key_state reads -- K in its operand order (one term), V with
// two consecutive keys per dword (one term), |k|^2 / 2 -- one wavefront per four keys, lane = coordinate.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void identity_pack_kernel(const uint16_t* K, const uint16_t* V, uint16_t* Kimg,
                                                            uint32_t* Vimg, float* nrm, int n, int d, int BH) {
    const int lane = threadIdx.x & 63;
    const long wid = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int groups_per_head = n / 4;
    if (wid >= (long)BH * groups_per_head) return;
    const int bh = (int)(wid / groups_per_head);
    const int r0 = 4 * (int)(wid % groups_per_head);
    float sq[4] = {0.f, 0.f, 0.f, 0.f};
    for (int t = lane; t < d; t += 64) {
        uint16_t kv[4], vv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long off = ((long)bh * n + r0 + e) * d + t;
            kv[e] = K[off];
            vv[e] = V[off];
            const float x = bf16_to_f32(kv[e]);
            sq[e] = fmaf(x, x, sq[e]);
            const int r = r0 + e;
            if (Kimg) {
                const long io = (long)bh * n * d +
                                ((((long)(r >> 5) * (d / 16) + (t >> 4)) * 2 + ((t >> 3) & 1)) * 32 + (r & 31)) * 8 + (t & 7);
                Kimg[io] = kv[e];
            }
        }
#pragma unroll
        for (int pr = 0; pr < 2; ++pr)
            Vimg[((long)bh * (n / 2) + r0 / 2 + pr) * d + t] = (uint32_t)vv[2 * pr] | ((uint32_t)vv[2 * pr + 1] << 16);
    }
    if (nrm) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float tot = wave_sum(sq[e]);
            if (lane == 0) nrm[(long)bh * n + r0 + e] = 0.5f * tot;
        }
    }
}

// p.k == p.n here: every position is a key.  Fills S, z, c in ctx and the St/zp/cw images.
flurka_status fast_identity_key_state(const Problem& p, const void* K, const void* V, const void* omega, float* S,
                                      float* z, float* c, const KeyStateBuffers& b, hipStream_t s) {
    const KeyStatePlan q = key_state_plan(p);
    {
        StageScope sc(s, STAGE_K_IDENTITY_PACK);
        const long waves = (long)p.BH * (p.n / 4);
        hipLaunchKernelGGL(identity_pack_kernel, grid1d(waves, 4), dim3(256), 0, s, (const uint16_t*)K, (const uint16_t*)V,
                           p.elu ? (uint16_t*)nullptr : b.Kimg, b.Vimg, p.elu ? (float*)nullptr : b.nrm, p.n, p.d, p.BH);
        FLURKA_CHECK_LAUNCH();
    }
    StageScope sc(s, STAGE_K_KEY_STATE);
    KeyStateArgs ka{};
    ka.Kimg = b.Kimg; ka.Kp = nullptr; ka.Kb = (const uint16_t*)K; ka.Vimg = b.Vimg; ka.nrm = b.nrm;
    ka.omega = (const uint16_t*)omega;
    ka.S = S; ka.z = z; ka.c = c;
    ka.St = b.St; ka.zp = b.zp; ka.cw = b.cw;
    ka.omega_head_stride = p.omega_per_head ? (long)p.m * p.d : 0;
    ka.BH = p.BH; ka.H = p.H; ka.k = p.k; ka.kpad = q.kpad; ka.mf = p.mf; ka.mfp = p.mfp;
    ka.FT = q.FT; ka.KR = q.KR; ka.tiles_per_range = q.tiles_per_range;
    return p.d == 64 ? launch_key_state<64>(p, ka, true, s) : launch_key_state<128>(p, ka, true, s);
}

}  // namespace flurka
