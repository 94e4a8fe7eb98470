// bf16 MFMA backward of the query side of FLuRKA attention (gfx950): dQ, dS, dz.
//
// Chain rule of out = (P S)/(P z) with P_ij = exp(u_ij + c_j - mu_i), u = Q omega^T (positive random
// features, Sec. 2 "Kernel Methods"; ratio form of App. D).  With the normalised weights
// W_ij = P_ij / D_i = exp(u_ij + c_j - lambda_i), lambda_i = mu_i + ln D_i, and g_i = G_i . out_i:
//     dU_ij = W_ij (G_i . S_j - g_i z_j)        dQ = dU omega
//     dS_j  = sum_i W_ij G_i                    dz_j = - sum_i W_ij g_i
// (the -rowsum(dU) q term of the feature map's derivative vanishes: sum_j dU_ij = 0 identically).
//
// Where attention is concentrated on few (key, feature) pairs these sums cancel almost completely:
// G_i . S_j - g_i z_j = z_j G_i . (S_j / z_j - out_i) with out_i close to S_j / z_j for the features that
// carry the weight, and likewise dPhiK_rj = sum_i W_ij (G_i . V'_r - g_i) on the key side.  A g_i taken
// from the rounded output (relative error 2^-9), or S rounded to one bf16 term, then leaves errors far
// larger than the result.  So:
//   * S_j / z_j enters as a two-term bf16 split (hi + lo), and b_ij = W_ij z_j is what is exponentiated
//     (c_j + ln z_j is the shift), so that r_ij = b_ij (G_i . S_j / z_j - ghat_i) is small where it cancels;
//   * ghat_i = G_i . out_i (rounded output) is only a first estimate: with sR_i = sum_j r_ij and
//     sB_i = sum_j b_ij (= 1 up to the rounding of the forward's lambda_i), g_i = ghat_i + sR_i / sB_i is
//     consistent with the weights this kernel uses, and
//         dQ_i = (sum_j r_ij omega_j - (sR_i / sB_i) sum_j b_ij omega_j) / sB_i
//     needs a second accumulator (sum_j b_ij omega_j) but no second pass;
//   * the dS kernel uses the renormalised lambda_i + ln sB_i and forms dz_j from the same bf16-rounded
//     weights that enter dS_j.
//
// Two kernels, both built on v_mfma_f32_32x32x16_bf16 with operands chained through registers:
//   bwd_query_x  one wavefront per 32 query rows, lane = query: lambda_i comes from the forward (ctx);
//                forms r^T and b^T tile by tile and accumulates the two parts of dQ^T
//   bwd_query_y  one wavefront per (head, 32 features, query range), lane = feature: recomputes W with
//                the renormalised lambda, accumulates dS and dz over its queries; a merge kernel sums ranges
// then bwd_key (dK', dV' from dS, dz) and the four sequence-length GEMMs of flurka_gemm.h.
// phi = elu + 1 has dQ and dS kernels of its own (bwd_query_x_elu, the ELU variant of bwd_query_y) and
// leaves the small key side to the generic kernels.
#include "flurka_fast.h"
#include "flurka_gemm.h"

namespace flurka {

#define FLURKA_CHECK_LAUNCH()                                   \
    do {                                                        \
        if (hipGetLastError() != hipSuccess) return FLURKA_ERR_LAUNCH; \
    } while (0)

static inline dim3 grid1d(long total, int block) { return dim3((unsigned)((total + block - 1) / block)); }

constexpr float LOG2E = FLURKA_LOG2E;

typedef short short4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 lds_read_tr16(const unsigned char* p) {
    const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
    return __builtin_bit_cast(uint2, v);
}

// ---------------------------------------------------------------------------
// bwd_query_x
// ---------------------------------------------------------------------------
struct BwdXArgs {
    const uint16_t* Q;
    const uint16_t* G;         // dOut
    const uint16_t* O;         // out
    const uint16_t* omega;     // (H|1, m, d)
    const float* S;            // ctx: (BH, mf, d), (BH, mf), (BH, mf)
    const float* z;
    const float* c;
    const float* lse;          // (BH, n)  lambda_i, written by the forward
    uint16_t* dQ;
    float* delta;              // (BH, n)  g_i
    float* lam2;               // (BH, n)  lambda_i + ln sB_i: the normaliser the dS kernel uses
    int n, H, mf, tiles_per_head;   // mf: features incl. the padding of a ragged last tile; tiles of 32 rows
    int mr;                         // features that exist (rows of omega, strides of S, z, c in ctx)
    long total_tiles;               // BH * tiles_per_head
    long omega_head_stride;    // 0 if shared
};

// LDS of a workgroup: omega (once: omega^T is read out of the same image with transposing loads, see
// bwd_query_y for their layout), the two terms of Sp, c', and -- head size 64 -- a 32 x D area per
// wavefront through which tiles cross between memory order and operand order.  Larger head sizes
// ("direct") move rows of Q, dOut, out, dQ between memory and registers directly, 16 bytes per lane
// and step.
// The omega image has unpadded rows; 16-byte chunk c of row r sits at chunk position c ^ swz(r):
//   256-byte rows (d = 128): swz(r) = 4*(r%4) + (r/4)%4
//   128-byte rows (d = 64):  swz(r) = 4*((r/2)%2) + (r/4)%4
// Either way 16 consecutive rows put the same chunk into 16 different bank groups (plain reads down a
// column of rows), and 4 consecutive rows put a 64-byte column group into 4 different quarters of the
// banks (transposing reads).
// RING (d = 128 with more features than all three images have room for): the lo terms of S/z are not
// resident; the wavefronts of a workgroup walk the feature tiles in step, and the 32 lo rows of the next
// tile are built from ctx into one of two LDS slots while the current tile is worked on (one barrier
// per feature tile).
template <int D, bool RING = false>
struct BwdXLds {
    static_assert(D == 64 || D == 128, "row swizzles are written for 128- and 256-byte rows");
    static_assert(!RING || D == 128, "the ring variant fills one slot with 512 threads x 16 bytes");
    static constexpr bool direct = D > 64;
    static constexpr int nw = 8;                     // wavefronts per workgroup: two per SIMD (the two
                                                     // accumulator sets leave no room for a third)
    static constexpr int w_pitch = D * 2;                                // omega rows
    static constexpr int sp_pitch = (D + 8) * 2;                         // Sp rows
    static __host__ __device__ int lo_rows(int mf) { return RING ? 64 : mf; }
    static __host__ __device__ int images(int mf) {
        return mf * w_pitch + mf * sp_pitch + lo_rows(mf) * sp_pitch + mf * 4;
    }
    static constexpr int scratch = direct ? 0 : 32 * D * 2;              // per wavefront: one 32-row tile
    static __host__ __device__ int total(int mf) { return images(mf) + nw * scratch + 16; }    // + tile counter
    static __host__ __device__ int swz(int r) {
        return D == 128 ? ((r & 3) << 2) | ((r >> 2) & 3) : (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
    }
};

constexpr int X_THREADS = 512;
template <int D, bool RING>
__global__ __launch_bounds__(X_THREADS) void bwd_query_x_kernel(BwdXArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    using L = BwdXLds<D, RING>;
    static_assert(L::nw * 64 == X_THREADS, "launch bounds");
    constexpr bool DIRECT = L::direct;
    constexpr int X_NW = L::nw;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int mf = a.mf;
    unsigned char* lw = lds;                              // omega    [feature][d], swizzled chunks
    unsigned char* lsh = lw + mf * L::w_pitch;            // Sp hi    [feature][t slot]
    unsigned char* lsl = lsh + mf * L::sp_pitch;          // Sp lo    (RING: two slots of 32 rows)
    float* lc = (float*)(lsl + L::lo_rows(mf) * L::sp_pitch);    // c'
    constexpr int KS = D / 16;      // reduction steps over d (also over the t slots of G)
    constexpr int TT = D / 32;      // 32-row tiles of dQ^T
    const int FT = mf / 32;

    // Resident grid: each workgroup takes an equal, contiguous share of all (head, 32-row tile) pairs
    // and walks it head by head, refilling the LDS image when the head changes.
    const long tile_begin = a.total_tiles * blockIdx.x / gridDim.x;
    const long tile_end = a.total_tiles * (blockIdx.x + 1) / gridDim.x;
    for (long seg = tile_begin; seg < tile_end;) {
    const int bh = (int)(seg / a.tiles_per_head);
    long seg_end = (long)(bh + 1) * a.tiles_per_head;
    if (seg_end > tile_end) seg_end = tile_end;
    if (seg != tile_begin) __syncthreads();          // every wavefront is done with the previous image
    // omega as it lies; S_j / z_j as two bf16 terms (hi + lo), 8 slots per chunk: the slots of dOut's
    // operand order (head size 64: slot 8h + e of a group of 16 holds t = 8*(e/4) + 4*h + e%4; direct:
    // t = slot); c + ln z in the accumulator order of a 32-feature tile
    // Features past mr (the padding of a ragged last tile) get c' = -inf: their weights b are exactly 0
    // and nothing of them reaches dQ, g or lambda; their rows of omega and S/z are those of the last
    // real feature (any finite values do: they only ever multiply that 0).
    const int mr = a.mr;
    const float* Sg = a.S + (long)bh * mr * D;
    const float* zg = a.z + (long)bh * mr;
    constexpr int cpr = D / 8;
    auto sp_terms = [&](int r, int q, uint4& hi4, uint4& lo4) {      // chunk q of feature row r
        if (r >= mr) r = mr - 1;
        const int t0 = DIRECT ? 8 * q : 16 * (q >> 1) + 4 * (q & 1);
        const float4 s0 = *(const float4*)(Sg + (long)r * D + t0);
        const float4 s1 = *(const float4*)(Sg + (long)r * D + t0 + (DIRECT ? 4 : 8));
        const float rz = 1.f / zg[r];
        const float v[8] = {s0.x * rz, s0.y * rz, s0.z * rz, s0.w * rz, s1.x * rz, s1.y * rz, s1.z * rz, s1.w * rz};
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split2_pair(v[2 * e], v[2 * e + 1], hi[e], lo[e]);
        hi4 = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        lo4 = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    };
    {
        const uint16_t* og = a.omega + (long)(bh % a.H) * a.omega_head_stride;
        for (int c = tid; c < mf * cpr; c += X_NW * 64) {
            const int r = c / cpr, q = c % cpr;
            *(uint4*)(lw + r * L::w_pitch + 16 * (q ^ L::swz(r))) = ld16(og + (long)(r < mr ? r : mr - 1) * D + 8 * q);
            uint4 hi, lo;
            sp_terms(r, q, hi, lo);
            *(uint4*)(lsh + r * L::sp_pitch + 16 * q) = hi;
            if constexpr (!RING) *(uint4*)(lsl + r * L::sp_pitch + 16 * q) = lo;
        }
        if constexpr (RING) {          // slot 0 <- feature tile 0
            uint4 hi, lo;
            sp_terms(tid / cpr, tid % cpr, hi, lo);
            *(uint4*)(lsl + (tid / cpr) * L::sp_pitch + 16 * (tid % cpr)) = lo;
        }
        const float* cg = a.c + (long)bh * mr;
        for (int slot = tid; slot < mf; slot += X_NW * 64) {
            const int g = slot & 15, h = (slot >> 4) & 1;
            const int f = (slot & ~31) + 8 * (g >> 2) + 4 * h + (g & 3);
            lc[slot] = f < mr ? cg[f] + logf(zg[f]) : -INFINITY;
        }
    }
    // tiles of the segment are handed out on demand (see query_stream_kernel): wavefront w starts with
    // tile w and takes the next free one from this counter whenever it finishes
    int* const next_tile = (int*)(lds + L::images(mf) + X_NW * L::scratch);
    if (tid == 0) *next_tile = X_NW;
    __syncthreads();

    const long head_off = (long)bh * a.n * D;
    const int row_begin = (int)(seg - (long)bh * a.tiles_per_head) * 32;
    int row_end = (int)(seg_end - (long)bh * a.tiles_per_head) * 32;
    if (row_end > a.n) row_end = a.n;
    seg = seg_end;

    // One tile = this lane's query row: Q as the B operand of u^T (8 consecutive d per step), dOut as
    // the B operand of (S/z) G^T, the same elements of out (for ghat_i) and lambda_i.
    // Head size 64: slots (h, j) of step s of dOut hold t = 16*s + 8*(j/4) + 4*h + j%4 (Sp is packed to
    // match).  Tiles move between memory and a wavefront-private 32 x D area of LDS as whole 16-byte
    // chunks in memory order (32 rows are one contiguous block: every wavefront instruction covers
    // 1 KiB of consecutive bytes), and between LDS and registers in the per-lane operand layouts.
    // Chunk c of row r sits at chunk position c ^ ((r >> 1) & 7): conflict-free both ways.
    // Direct: dOut and out are taken like Q.  (n is a multiple of 32 on this path: tiles are whole.)
    constexpr int CPR = D / 8, ROWB = D * 2, LPT = 32 * CPR / 64;
    unsigned char* const scr = lds + L::images(mf) + wave * L::scratch;
    auto scr_at = [&](int row, int c) -> unsigned char* { return scr + row * ROWB + 16 * (c ^ ((row >> 1) & 7)); };
    struct Tile { uint4 q[KS], g[KS]; float lam, gh; };
    auto dot2 = [](uint32_t x, uint32_t y, float acc) {
        acc = fmaf(bf16_to_f32((uint16_t)(x & 0xffffu)), bf16_to_f32((uint16_t)(y & 0xffffu)), acc);
        return fmaf(bf16_to_f32((uint16_t)(x >> 16)), bf16_to_f32((uint16_t)(y >> 16)), acc);
    };
    auto dot8 = [&](const uint4& x, const uint4& y, float acc) {
        acc = dot2(x.x, y.x, acc); acc = dot2(x.y, y.y, acc);
        acc = dot2(x.z, y.z, acc); return dot2(x.w, y.w, acc);
    };
    // loads one tile; ghat = G_i . out_i over the elements this half of the wavefront holds
    auto load_tile = [&](int row0, Tile& t) {
        float gd = 0.f;
        if constexpr (DIRECT) {
            const long off = head_off + (long)(row0 + l32) * D + 8 * half;
            uint4 o[KS];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                t.q[s] = ld16(a.Q + off + 16 * s);
                t.g[s] = ld16(a.G + off + 16 * s);
                o[s] = ld16(a.O + off + 16 * s);
            }
            t.lam = a.lse[(long)bh * a.n + row0 + l32];
#pragma unroll
            for (int s = 0; s < KS; ++s) gd = dot8(t.g[s], o[s], gd);
        } else {
            uint4 rq[LPT], rg[LPT], ro[LPT];
            const long off = head_off + (long)row0 * D + 8 * lane;
#pragma unroll
            for (int u = 0; u < LPT; ++u) {
                rq[u] = ld16(a.Q + off + 512 * u);
                rg[u] = ld16(a.G + off + 512 * u);
                ro[u] = ld16(a.O + off + 512 * u);
            }
            t.lam = a.lse[(long)bh * a.n + row0 + l32];
#pragma unroll
            for (int u = 0; u < LPT; ++u) *(uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR) = rq[u];
#pragma unroll
            for (int s = 0; s < KS; ++s) t.q[s] = *(const uint4*)scr_at(l32, 2 * s + half);
#pragma unroll
            for (int u = 0; u < LPT; ++u) *(uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR) = rg[u];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint2 g0 = *(const uint2*)(scr_at(l32, 2 * s) + 8 * half);
                const uint2 g1 = *(const uint2*)(scr_at(l32, 2 * s + 1) + 8 * half);
                t.g[s] = make_uint4(g0.x, g0.y, g1.x, g1.y);
            }
#pragma unroll
            for (int u = 0; u < LPT; ++u) *(uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR) = ro[u];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint2 o0 = *(const uint2*)(scr_at(l32, 2 * s) + 8 * half);
                const uint2 o1 = *(const uint2*)(scr_at(l32, 2 * s + 1) + 8 * half);
                gd = dot8(t.g[s], make_uint4(o0.x, o0.y, o1.x, o1.y), gd);
            }
        }
        t.gh = half_sum(gd);
    };
    // this lane's byte offsets into the omega image
    //   plain reads (A operand of u^T): row 32*ft + l32, chunk 2*s + half
    //   transposing reads (A operand of dQ^T, column t = 32*tt + l32 of 8 features): this lane supplies
    //   row 4*half + s16/4 (+ 8 for the second read) of a 16-feature group, 8 bytes at column
    //   16*(lane/16 % 2) + 4*(s16 % 4) of the 32-column group tt
    const int s16 = lane & 15, r4 = s16 >> 2;
    const int u_lane = l32 * L::w_pitch, u_xor = 16 * (L::swz(l32) ^ half);
    const int tr_row = (4 * half + r4) * L::w_pitch + 8 * (s16 & 1);
    const int tr_low0 = 16 * ((2 * ((lane >> 4) & 1) + ((s16 >> 1) & 1)) ^ half);     // first read; second: ^ 32
    const int tr_hi = D == 128 ? r4 : (r4 >> 1);                                      // XORed with tt

    // per-tile state: r^T and b^T tile by tile; accR = omega^T r^T, accB = omega^T b^T
    Tile cur;
    floatx16 accR[TT], accB[TT];
    float sR = 0.f, sB = 0.f, nlam = 0.f, gh = 0.f;
    auto begin_tile = [&](int row0) {
        load_tile(row0, cur);
#pragma unroll
        for (int t = 0; t < TT; ++t) { accR[t] = zero16(); accB[t] = zero16(); }
        sR = 0.f; sB = 0.f;
        nlam = -cur.lam * LOG2E;
        gh = cur.gh;
    };
    // one feature tile; lo_rows: the 32 rows of the lo term of S/z that belong to it
    auto feature_tile = [&](int ft, const unsigned char* lo_rows) {
        floatx16 u, tp = zero16();                           // tp: T'^T tile, G_i . S_j / z_j
        const float4* ct = (const float4*)(lc + 32 * ft + 16 * half);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = ct[q];
            u[4 * q] = v.x; u[4 * q + 1] = v.y; u[4 * q + 2] = v.z; u[4 * q + 3] = v.w;
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            u = mfma32(*(const uint4*)(lw + 32 * ft * L::w_pitch + u_lane + ((32 * s) ^ u_xor)), cur.q[s], u);
            const int so = l32 * L::sp_pitch + 32 * s + 16 * half;
            tp = mfma32(*(const uint4*)(lsh + 32 * ft * L::sp_pitch + so), cur.g[s], tp);
            tp = mfma32(*(const uint4*)(lo_rows + so), cur.g[s], tp);
        }
        uint32_t pr[8], pb[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const float b0 = fast_exp2(fmaf(u[2 * q], LOG2E, nlam));
            const float b1 = fast_exp2(fmaf(u[2 * q + 1], LOG2E, nlam));
            pb[q] = pack_bf16(b0, b1);
            pr[q] = pack_bf16(b0 * (tp[2 * q] - gh), b1 * (tp[2 * q + 1] - gh));
            sB = add_bf16_pair(pb[q], sB);
            sR = add_bf16_pair(pr[q], sR);
        }
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
            const uint4 rb = {pr[4 * sp], pr[4 * sp + 1], pr[4 * sp + 2], pr[4 * sp + 3]};
            const uint4 bb = {pb[4 * sp], pb[4 * sp + 1], pb[4 * sp + 2], pb[4 * sp + 3]};
            const unsigned char* fb = lw + (32 * ft + 16 * sp) * L::w_pitch + tr_row;
#pragma unroll
            for (int t = 0; t < TT; ++t) {
                const int col = ((t ^ tr_hi) << 6) + tr_low0;
                const uint2 w0 = lds_read_tr16(fb + col);
                const uint2 w1 = lds_read_tr16(fb + 8 * L::w_pitch + (col ^ 32));
                const uint4 wt = make_uint4(w0.x, w0.y, w1.x, w1.y);
                accR[t] = mfma32(wt, rb, accR[t]);
                accB[t] = mfma32(wt, bb, accB[t]);
            }
        }
    };
    auto end_tile = [&](int row0) {
        const int qrow = row0 + l32;
        // this row's normaliser and the correction of ghat; both halves of the wavefront hold the same row
        const float tR = half_sum(sR), tB = half_sum(sB);
        const float inv = 1.f / tB;
        const float dg = tR * inv;
        if (half == 0) {
            a.delta[(long)bh * a.n + qrow] = gh + dg;
            a.lam2[(long)bh * a.n + qrow] = cur.lam + logf(tB);
        }
        // dQ rows: 16-byte pieces; head size 64 passes them through the transposition area so that whole
        // chunks leave in memory order
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int q = 0; q < 4; q += 2) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = (accR[t][4 * q + e] - dg * accB[t][4 * q + e]) * inv;
                uint2 ev, od;
                ev.x = pack_bf16(v[0], v[1]); ev.y = pack_bf16(v[2], v[3]);
                od.x = pack_bf16(v[4], v[5]); od.y = pack_bf16(v[6], v[7]);
                const uint4 piece = join_halves(ev, od);
                if constexpr (DIRECT) *(uint4*)(a.dQ + head_off + (long)qrow * D + 8 * (4 * t + q + half)) = piece;
                else                  *(uint4*)scr_at(l32, 4 * t + q + half) = piece;
            }
        if constexpr (!DIRECT) {
            uint16_t* ob = a.dQ + head_off + (long)row0 * D + 8 * lane;
#pragma unroll
            for (int u = 0; u < LPT; ++u)
                *(uint4*)(ob + 512 * u) = *(const uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR);
        }
    };

    if constexpr (!RING) {
        for (int row0 = row_begin + 32 * wave; row0 < row_end;) {
            int grabbed = 0;
            if (lane == 0) grabbed = atomicAdd(next_tile, 1);
            const int row_next = row_begin + 32 * __builtin_amdgcn_readfirstlane(grabbed);
            begin_tile(row0);
            for (int ft = 0; ft < FT; ++ft) feature_tile(ft, lsl + 32 * ft * L::sp_pitch);
            end_tile(row0);
            row0 = row_next;
        }
    } else {
        // Rounds of X_NW tiles, one per wavefront; every wavefront runs every iteration (also without a
        // tile in the last round), so the barriers match.  Iteration (round, ft) reads ring slot `slot`
        // and fills the other one for the next iteration; the barrier at the top of an iteration makes
        // that fill visible and separates it from the reads of the slot it will overwrite next.
        const int ntiles = (row_end - row_begin) / 32;
        const int fr = tid / cpr, fq = tid % cpr;            // this thread's chunk of a 32-row slot
        int slot = 0;
        for (int base = 0; base < ntiles; base += X_NW) {
            const bool has = base + wave < ntiles;
            const int row0 = row_begin + 32 * (has ? base + wave : 0);
            if (has) begin_tile(row0);
            for (int ft = 0; ft < FT; ++ft) {
                if (base != 0 || ft != 0) __syncthreads();
                uint4 nhi, nlo;
                sp_terms(32 * (ft + 1 < FT ? ft + 1 : 0) + fr, fq, nhi, nlo);
                if (has) feature_tile(ft, lsl + 32 * slot * L::sp_pitch);
                *(uint4*)(lsl + (32 * (slot ^ 1) + fr) * L::sp_pitch + 16 * fq) = nlo;
                slot ^= 1;
            }
            if (has) end_tile(row0);
        }
    }
    }   // head segments
}

// ---------------------------------------------------------------------------
// bwd_query_x for phi = elu + 1 (the "RNN" feature map of Sec. 2; features = the d coordinates):
//     P_ij = elu(q_ij) + 1,  D_i = P_i . z,  T_ij = G_i . S_j,  g_i = (P_i . T_i) / D_i  (= G_i . out_i),
//     dQ_ij = (T_ij - g_i z_j) / D_i * phi'(q_ij),  phi'(x) = 1 (x > 0), exp(x) otherwise.
// One contraction (T, with S as a two-term bf16 split so that T_ij - g_i z_j keeps fp32 accuracy where
// it cancels); everything else is elementwise in the accumulator layout, so Q and dOut are both taken in
// the accumulator's slot order (slot 8h + e of a group of 16 holds t = 8*(e/4) + 4*h + e%4).  g_i and
// 1/D_i go to the dS kernel.
// ---------------------------------------------------------------------------
struct BwdXEluArgs {
    const uint16_t* Q;
    const uint16_t* G;         // dOut
    const float* S;            // ctx (BH, d, d): S[j][t]
    const float* z;            // ctx (BH, d)
    uint16_t* dQ;
    float* delta;              // (BH, n)  g_i
    float* dinv;               // (BH, n)  1 / D_i
    int n, tiles_per_head;
    long total_tiles;
};

template <int D>
struct BwdXEluLds {
    static constexpr bool direct = D > 64;
    static constexpr int nw = 8;
    static constexpr int sp_pitch = (D + 8) * 2;
    static constexpr int images = 2 * D * sp_pitch + D * 4;              // S hi, S lo, z
    static constexpr int scratch = direct ? 0 : 32 * D * 2;
    static constexpr int total = images + nw * scratch + 16;
};

__device__ __forceinline__ float elu1_of(float x) { return x > 0.f ? x + 1.f : __expf(x); }

template <int D>
__global__ __launch_bounds__(512) void bwd_query_x_elu_kernel(BwdXEluArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    using L = BwdXEluLds<D>;
    constexpr bool DIRECT = L::direct;
    constexpr int X_NW = L::nw;
    constexpr int KS = D / 16, TT = D / 32;         // TT feature tiles = coordinate tiles
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    unsigned char* lsh = lds;
    unsigned char* lsl = lsh + D * L::sp_pitch;
    float* lz = (float*)(lsl + D * L::sp_pitch);    // z in accumulator order of a 32-feature tile
    int* const next_tile = (int*)(lds + L::images + X_NW * L::scratch);

    const long tile_begin = a.total_tiles * blockIdx.x / gridDim.x;
    const long tile_end = a.total_tiles * (blockIdx.x + 1) / gridDim.x;
    for (long seg = tile_begin; seg < tile_end;) {
    const int bh = (int)(seg / a.tiles_per_head);
    long seg_end = (long)(bh + 1) * a.tiles_per_head;
    if (seg_end > tile_end) seg_end = tile_end;
    if (seg != tile_begin) __syncthreads();
    {
        const float* Sg = a.S + (long)bh * D * D;
        constexpr int cpr = D / 8;
        for (int c = tid; c < D * cpr; c += X_NW * 64) {
            const int r = c / cpr, q = c % cpr;
            const int t0 = 16 * (q >> 1) + 4 * (q & 1);
            const float4 s0 = *(const float4*)(Sg + (long)r * D + t0);
            const float4 s1 = *(const float4*)(Sg + (long)r * D + t0 + 8);
            const float v[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) split2_pair(v[2 * e], v[2 * e + 1], hi[e], lo[e]);
            *(uint4*)(lsh + r * L::sp_pitch + 16 * q) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            *(uint4*)(lsl + r * L::sp_pitch + 16 * q) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
        const float* zg = a.z + (long)bh * D;
        for (int slot = tid; slot < D; slot += X_NW * 64) {
            const int g = slot & 15, h = (slot >> 4) & 1;
            lz[slot] = zg[(slot & ~31) + 8 * (g >> 2) + 4 * h + (g & 3)];
        }
    }
    if (tid == 0) *next_tile = X_NW;
    __syncthreads();

    const long head_off = (long)bh * a.n * D;
    const int row_begin = (int)(seg - (long)bh * a.tiles_per_head) * 32;
    int row_end = (int)(seg_end - (long)bh * a.tiles_per_head) * 32;
    if (row_end > a.n) row_end = a.n;
    seg = seg_end;

    constexpr int CPR = D / 8, ROWB = D * 2, LPT = 32 * CPR / 64;
    unsigned char* const scr = lds + L::images + wave * L::scratch;
    auto scr_at = [&](int row, int c) -> unsigned char* { return scr + row * ROWB + 16 * (c ^ ((row >> 1) & 7)); };
    // this lane's row of Q and of dOut in accumulator slot order (see bwd_query_x_kernel for the staging)
    uint4 qv[KS], gv[KS];
    auto load_tile = [&](int row0) {
        if constexpr (DIRECT) {
            const long off = head_off + (long)(row0 + l32) * D + 4 * half;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint2 q0 = *(const uint2*)(a.Q + off + 16 * s), q1 = *(const uint2*)(a.Q + off + 16 * s + 8);
                const uint2 g0 = *(const uint2*)(a.G + off + 16 * s), g1 = *(const uint2*)(a.G + off + 16 * s + 8);
                qv[s] = make_uint4(q0.x, q0.y, q1.x, q1.y);
                gv[s] = make_uint4(g0.x, g0.y, g1.x, g1.y);
            }
        } else {
            uint4 rq[LPT], rg[LPT];
            const long off = head_off + (long)row0 * D + 8 * lane;
#pragma unroll
            for (int u = 0; u < LPT; ++u) {
                rq[u] = ld16(a.Q + off + 512 * u);
                rg[u] = ld16(a.G + off + 512 * u);
            }
#pragma unroll
            for (int u = 0; u < LPT; ++u) *(uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR) = rq[u];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint2 x0 = *(const uint2*)(scr_at(l32, 2 * s) + 8 * half);
                const uint2 x1 = *(const uint2*)(scr_at(l32, 2 * s + 1) + 8 * half);
                qv[s] = make_uint4(x0.x, x0.y, x1.x, x1.y);
            }
#pragma unroll
            for (int u = 0; u < LPT; ++u) *(uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR) = rg[u];
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint2 x0 = *(const uint2*)(scr_at(l32, 2 * s) + 8 * half);
                const uint2 x1 = *(const uint2*)(scr_at(l32, 2 * s + 1) + 8 * half);
                gv[s] = make_uint4(x0.x, x0.y, x1.x, x1.y);
            }
        }
    };

    for (int row0 = row_begin + 32 * wave; row0 < row_end;) {
        const int qrow = row0 + l32;
        int grabbed = 0;
        if (lane == 0) grabbed = atomicAdd(next_tile, 1);
        const int row_next = row_begin + 32 * __builtin_amdgcn_readfirstlane(grabbed);
        load_tile(row0);

        // T^T tiles: rows = features j (accumulator element g <-> j = 32*ft + 8*(g/4) + 4*half + g%4)
        floatx16 tp[TT];
#pragma unroll
        for (int ft = 0; ft < TT; ++ft) {
            tp[ft] = zero16();
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int so = (32 * ft + l32) * L::sp_pitch + 32 * s + 16 * half;
                tp[ft] = mfma32(*(const uint4*)(lsh + so), gv[s], tp[ft]);
                tp[ft] = mfma32(*(const uint4*)(lsl + so), gv[s], tp[ft]);
            }
        }
        // P, D, g in the same layout: element g of tile ft is slot g % 8 of step 2*ft + g / 8
        float pv[TT][16], zv[TT][16];
        float dsum = 0.f, gsum = 0.f;
#pragma unroll
        for (int ft = 0; ft < TT; ++ft)
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const uint4& w4 = qv[2 * ft + (g >> 3)];
                const uint32_t w = (g & 7) < 2 ? w4.x : (g & 7) < 4 ? w4.y : (g & 7) < 6 ? w4.z : w4.w;
                const float q = (g & 1) ? pair_hi(w) : pair_lo(w);
                const float p = elu1_of(q);
                const float zz = lz[32 * ft + 16 * half + g];
                dsum = fmaf(p, zz, dsum);
                gsum = fmaf(p, tp[ft][g], gsum);
                pv[ft][g] = q > 0.f ? 1.f : p;              // phi'(q)
                zv[ft][g] = zz;
            }
        dsum = half_sum(dsum);
        gsum = half_sum(gsum);
        const float inv = 1.f / dsum;
        const float gi = gsum * inv;
        if (half == 0) {
            a.delta[(long)bh * a.n + qrow] = gi;
            a.dinv[(long)bh * a.n + qrow] = inv;
        }
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int q = 0; q < 4; q += 2) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = (tp[t][4 * q + e] - gi * zv[t][4 * q + e]) * inv * pv[t][4 * q + e];
                uint2 ev, od;
                ev.x = pack_bf16(v[0], v[1]); ev.y = pack_bf16(v[2], v[3]);
                od.x = pack_bf16(v[4], v[5]); od.y = pack_bf16(v[6], v[7]);
                const uint4 piece = join_halves(ev, od);
                if constexpr (DIRECT) *(uint4*)(a.dQ + head_off + (long)qrow * D + 8 * (4 * t + q + half)) = piece;
                else                  *(uint4*)scr_at(l32, 4 * t + q + half) = piece;
            }
        if constexpr (!DIRECT) {
            uint16_t* ob = a.dQ + head_off + (long)row0 * D + 8 * lane;
#pragma unroll
            for (int u = 0; u < LPT; ++u)
                *(uint4*)(ob + 512 * u) = *(const uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR);
        }
        row0 = row_next;
    }
    }   // head segments
}

// ---------------------------------------------------------------------------
// bwd_query_y: one wavefront per (head, feature tile, query range)
// ---------------------------------------------------------------------------
struct BwdYArgs {
    const uint16_t* Q;
    const uint16_t* G;
    const uint16_t* omega;
    const float* c;            // ctx shifts, natural order (BH, mf)
    const float* lse;          // renormalised lambda_i from bwd_query_x; elu1: 1 / D_i
    const float* delta;
    float* dSpart;             // (BH, R, mf, d)
    float* dzpart;             // (BH, R, mf)
    long omega_head_stride;
    int BH, H, n, mf, FT, R, tiles_per_range;   // mf incl. the padding of a ragged last feature tile
    int mr;                                     // features that exist (rows of omega, stride of c)
};

// A workgroup is NW wavefronts = NW feature tiles of one (head, query range).  They need the same
// Q rows (A operand of u = Q omega^T) and the same dOut rows (B operand of dS = W^T dOut, contraction
// over queries), so blocks of Y_ST 32-query tiles are loaded once per workgroup with 16-byte loads and
// kept in LDS row-major.  The B operand needs, per lane, one column t of dOut for 8 query rows: that is
// what ds_read_b64_tr_b16 delivers from a row-major tile.  Layout of that instruction (checked on
// hardware): in each group of 16 lanes, lane s supplies the address of 4 consecutive 16-bit elements
// M[s][0..3]; lane i receives M[4j + i/4][i%4], j = 0..3.  With lane s pointing at row s/4, columns
// 4*(s%4).. of a 4 x 16 block, lane i receives column i of the block's four rows.
// The next block is requested into registers while the current one is worked on.
constexpr int Y_ST = 4;

// elu1: W_ij = (elu(q_ij) + 1) / D_i needs no contraction; the Q tile is read through the same
// transposing loads as the dOut tile (lane = feature), so it gets that tile's pitch.
template <int D, bool ELU = false>
struct BwdYLds {
    static constexpr int rows = 32 * Y_ST;
    static constexpr int g_pitch = D * 2 + 64;       // 4 consecutive rows fall into 4 distinct bank groups
    static constexpr int q_pitch = ELU ? g_pitch : (D + 8) * 2;   // plain: conflict-free 16-byte reads down a column of rows
    static constexpr int total = rows * (q_pitch + g_pitch) + 2 * rows * 4;
};


template <int D, int NW, bool ELU>
__global__ __launch_bounds__(NW * 64) void bwd_query_y_kernel(BwdYArgs a) {
    constexpr int KS = D / 16, TT = D / 32;
    using L = BwdYLds<D, ELU>;
    constexpr int QP = L::q_pitch, GP = L::g_pitch, ROWS = L::rows;
    constexpr int CPR = D / 8;                 // 16-byte chunks per row
    constexpr int NT = NW * 64;
    constexpr int LPT = ROWS * CPR / NT;       // 16-byte loads per thread per tensor per block
    static_assert(2 * ROWS <= NT && (ROWS * CPR) % NT == 0, "one lambda or g value per thread");
    extern __shared__ __attribute__((aligned(16))) unsigned char sm[];
    unsigned char* qs = sm;
    unsigned char* gs = sm + ROWS * QP;
    float* ll = (float*)(gs + ROWS * GP);      // lambda_i * log2(e); +inf past the end of the range
    float* ld = ll + ROWS;                     // g_i
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int FG = (a.FT + NW - 1) / NW;
    int id = blockIdx.x;
    const int fg = id % FG; id /= FG;
    const int r = id % a.R;
    const int bh = id / a.R;
    const int ft = NW * fg + wave;
    const bool active = ft < a.FT;
    const int ftc = active ? ft : a.FT - 1;
    const int QTn = a.n / 32;
    const int qt0 = r * a.tiles_per_range;
    int qt1 = qt0 + a.tiles_per_range;
    if (qt1 > QTn) qt1 = QTn;
    const int row_last = 32 * qt1 - 1;
    const long head_off = (long)bh * a.n * D;
    const long vec_off = (long)bh * a.n;

    uint4 wf[KS];
    float cj = 0.f;
    if constexpr (!ELU) {
        // a feature of the padding (ragged last tile): c = -inf, so its weights and its rows of dS, dz are
        // exactly 0; its omega row is the last real feature's (any finite row does)
        const int f = 32 * ftc + l32, fr = f < a.mr ? f : a.mr - 1;
        const uint16_t* og = a.omega + (long)(bh % a.H) * a.omega_head_stride + (long)fr * D + 8 * half;
#pragma unroll
        for (int s = 0; s < KS; ++s) wf[s] = ld16(og + 16 * s);
        cj = f < a.mr ? a.c[(long)bh * a.mr + fr] * LOG2E : -INFINITY;
    }
    floatx16 accS[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) accS[t] = zero16();
    float dz = 0.f;

    uint4 rq[LPT], rg[LPT];
    float rv = 0.f;                            // threads 0..ROWS-1: lambda, ROWS..2*ROWS-1: g
    auto load_block = [&](int qt) {
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            const int chunk = tid + NT * u;
            int row = 32 * qt + chunk / CPR;
            if (row > row_last) row = row_last;
            const long off = head_off + (long)row * D + 8 * (chunk % CPR);
            rq[u] = ld16(a.Q + off);
            rg[u] = ld16(a.G + off);
        }
        if (tid < 2 * ROWS) {
            const int row = 32 * qt + (tid % ROWS);
            if (tid < ROWS) rv = row <= row_last ? a.lse[vec_off + row] * (ELU ? 1.f : LOG2E) : (ELU ? 0.f : INFINITY);
            else            rv = row <= row_last ? a.delta[vec_off + row] : 0.f;
        }
    };
    auto store_block = [&]() {
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            const int chunk = tid + NT * u;
            const int row = chunk / CPR, c = chunk % CPR;
            *(uint4*)(qs + row * QP + 16 * c) = rq[u];
            *(uint4*)(gs + row * GP + 16 * c) = rg[u];
        }
        if (tid < 2 * ROWS) ll[tid] = rv;       // ld follows ll
    };

    // this lane's part of the transposing reads: row s/4 (+ 4*half) of a 4-row group, columns 4*(s%4)..
    // of the 16-column group (l32/16); see the layout note above
    const int s16 = lane & 15;
    const unsigned char* gtr = gs + (4 * half + (s16 >> 2)) * GP + 2 * (16 * ((lane >> 4) & 1) + 4 * (s16 & 3));
    const unsigned char* qtr = qs + (4 * half + (s16 >> 2)) * QP + 2 * (16 * ((lane >> 4) & 1) + 4 * (s16 & 3));

    if (qt0 < qt1) load_block(qt0);
    for (int qt = qt0; qt < qt1; qt += Y_ST) {
        store_block();
        __syncthreads();
        if (qt + Y_ST < qt1) load_block(qt + Y_ST);
#pragma unroll
        for (int i = 0; i < Y_ST; ++i) {
            // u tile: rows = queries of tile i, columns = this wavefront's features
            // (elu1: the same elements of Q itself, column 32*ft + l32, through transposing reads)
            floatx16 u = zero16();
            if constexpr (!ELU) {
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    u = mfma32(*(const uint4*)(qs + (32 * i + l32) * QP + 32 * s + 16 * half), wf[s], u);
            } else {
#pragma unroll
                for (int sp = 0; sp < 2; ++sp) {
                    const unsigned char* bp = qtr + (32 * i + 16 * sp) * QP + 64 * ftc;
                    const uint2 b0 = lds_read_tr16(bp);
                    const uint2 b1 = lds_read_tr16(bp + 8 * QP);
                    const uint32_t w[4] = {b0.x, b0.y, b1.x, b1.y};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        u[8 * sp + 2 * e] = elu1_of(pair_lo(w[e]));
                        u[8 * sp + 2 * e + 1] = elu1_of(pair_hi(w[e]));
                    }
                }
            }
            // element g <-> query 32*i + 8*(g/4) + 4*half + g%4
            uint32_t wk[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 lv = *(const float4*)(ll + 32 * i + 8 * q + 4 * half);
                const float4 dv = *(const float4*)(ld + 32 * i + 8 * q + 4 * half);
                float w0, w1, w2, w3;
                if constexpr (!ELU) {
                    w0 = fast_exp2(fmaf(u[4 * q], LOG2E, cj - lv.x));
                    w1 = fast_exp2(fmaf(u[4 * q + 1], LOG2E, cj - lv.y));
                    w2 = fast_exp2(fmaf(u[4 * q + 2], LOG2E, cj - lv.z));
                    w3 = fast_exp2(fmaf(u[4 * q + 3], LOG2E, cj - lv.w));
                } else {
                    w0 = u[4 * q] * lv.x; w1 = u[4 * q + 1] * lv.y; w2 = u[4 * q + 2] * lv.z; w3 = u[4 * q + 3] * lv.w;
                }
                wk[2 * q] = pack_bf16(w0, w1);
                wk[2 * q + 1] = pack_bf16(w2, w3);
                // dz from the rounded weights, the ones dS is formed with: dS_j . v'_r + dz_j then cancels
                // term by term where it should
                dz = fmaf(-__uint_as_float(wk[2 * q] << 16), dv.x, dz);
                dz = fmaf(-__uint_as_float(wk[2 * q] & 0xffff0000u), dv.y, dz);
                dz = fmaf(-__uint_as_float(wk[2 * q + 1] << 16), dv.z, dz);
                dz = fmaf(-__uint_as_float(wk[2 * q + 1] & 0xffff0000u), dv.w, dz);
            }
            // W^T tile as A operand (row = this lane's feature; slot 8h + e of step sp <-> query
            // 16*sp + 8*(e/4) + 4*h + e%4).  B operand: column t = 32*tt + l32 of the same queries.
            const uint4 wa[2] = {{wk[0], wk[1], wk[2], wk[3]}, {wk[4], wk[5], wk[6], wk[7]}};
#pragma unroll
            for (int sp = 0; sp < 2; ++sp)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const unsigned char* bp = gtr + (32 * i + 16 * sp) * GP + 64 * tt;
                    const uint2 b0 = lds_read_tr16(bp);
                    const uint2 b1 = lds_read_tr16(bp + 8 * GP);
                    accS[tt] = mfma32(wa[sp], make_uint4(b0.x, b0.y, b1.x, b1.y), accS[tt]);
                }
        }
        __syncthreads();
    }
    if (!active) return;
    dz = half_sum(dz);
    const long po = ((long)bh * a.R + r) * a.mf;
    if (half == 0) a.dzpart[po + 32 * ft + l32] = dz;
    float* sp = a.dSpart + po * D;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            const int f = 32 * ft + 8 * (g >> 2) + 4 * half + (g & 3);
            sp[(long)f * D + 32 * tt + l32] = accS[tt][g];
        }
}


// Sums the query ranges of dS, dz and writes the operand images of the key-side kernel:
//   dSimg  2 x (BH, mf, d) bf16 (hi, lo)    A operand of dPhiK^T = dS V'^T, and (through transposing
//                                           LDS reads) B operand of dV' = PhiK dS
//   dz     (BH, mf) fp32
// (elu1: the key side runs on the generic kernels and wants dS itself, fp32, instead of the image.)
__global__ void bwd_merge_kernel(uint16_t* dSimg, float* dS32, float* dz, const float* dSpart,
                                 const float* dzpart, int R, int mf, int d, long total) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;    // (bh, feature pair, t)
    if (idx >= total) return;
    const int t = (int)(idx % d);
    const long rest = idx / d;
    const int pr = (int)(rest % (mf / 2));
    const long bh = rest / (mf / 2);
    float s0 = 0.f, s1 = 0.f;
    for (int r = 0; r < R; ++r) {
        const float* p = dSpart + ((bh * R + r) * mf + 2 * pr) * d + t;
        s0 += p[0];
        s1 += p[d];
    }
    const long i0 = (bh * mf + 2 * pr) * d + t;
    if (dS32) {
        dS32[i0] = s0; dS32[i0 + d] = s1;
    } else {
        uint32_t hp, lp;
        split2_pair(s0, s1, hp, lp);
        const uint16_t h0 = (uint16_t)hp, h1 = (uint16_t)(hp >> 16), l0 = (uint16_t)lp, l1 = (uint16_t)(lp >> 16);
        const long plane = total * 2;                     // BH * mf * d
        dSimg[i0] = h0; dSimg[i0 + d] = h1;
        dSimg[plane + i0] = l0; dSimg[plane + i0 + d] = l1;
    }
    if (t == 0) {
        float z0 = 0.f, z1 = 0.f;
        for (int r = 0; r < R; ++r) {
            z0 += dzpart[(bh * R + r) * mf + 2 * pr];
            z1 += dzpart[(bh * R + r) * mf + 2 * pr + 1];
        }
        dz[bh * mf + 2 * pr] = z0;
        dz[bh * mf + 2 * pr + 1] = z1;
    }
}

// ---------------------------------------------------------------------------
// bwd_key: one wavefront per (head, 32 keys), lane = key.  Recomputes PhiK^T = exp(e^T - c) tile by
// tile with the forward's split-precision exponent, then
//     dPhiK^T = dS V'^T + dz 1^T       dUk = dPhiK * PhiK       rs_r = sum_j dUk_rj
//     dV' = PhiK dS                    dK' = dUk omega - rs_r k'_r
// with PhiK and dUk taken from the accumulator registers as A operands.  Every operand that enters a
// product whose result is later differenced is a two- or three-term bf16 split (fp32-level accuracy);
// the results leave as the bf16 images the two gradient GEMMs read.
// ---------------------------------------------------------------------------
struct BwdKeyArgs {
    const float* Kp; const float* Vp; const float* c;      // ctx
    const uint16_t* omega;
    const uint16_t* dSimg; const float* dz;
    uint16_t* img;     // 2 x (BH, kp, d): dK' then dV'
    uint16_t* imgT;    // 2 x (BH * d, kp)
    long omega_head_stride;
    int BH, H, k, kp, mf;   // mf incl. the padding of a ragged last feature tile (strides of dSimg, dz)
    int mr;                 // features that exist (rows of omega, stride of c)
};

// One workgroup per (head, 32 keys); its four wavefronts take every fourth feature tile and add their
// partial dV', dK', rs through LDS (fixed order, so the result does not depend on timing).
// The B operands of dV' = PhiK dS and dK' = dUk omega need, per lane, one column t for 8 features:
// each wavefront copies the 32 x d tiles of omega and dS (hi, lo) of its feature tile into its own
// LDS area with 16-byte loads and takes them out with ds_read_b64_tr_b16 (see bwd_query_y).
template <int D>
struct BwdKeyLds {
    static constexpr int pitch = D * 2 + 64;                       // as the dOut tile of bwd_query_y
    static constexpr int tile = 32 * pitch;
    static constexpr int tiles = 4 * 3 * tile;                     // per wavefront: omega, dS hi, dS lo
    static constexpr int slots = 4 * (2 * (D / 32) * 16 * 64 + 64) * 4;
    static constexpr int total = tiles > slots ? tiles : slots;    // the sums reuse the tile area
};

template <int D>
__global__ __launch_bounds__(256, D == 64 ? 2 : 1) void bwd_key_kernel(BwdKeyArgs a) {
    constexpr int KS = D / 16, TT = D / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
    const int wave = threadIdx.x >> 6;
    const int KT = a.kp / 32;
    // the KT workgroups of one head read the same omega and dS images: ids equal mod 8 = one XCD, one L2
    const int slot = (int)(blockIdx.x >> 3);
    const int kt = slot % KT;
    const int bh = (slot / KT) * 8 + (int)(blockIdx.x & 7);
    if (bh >= a.BH) return;                                // head count rounded up to whole groups of 8
    const int FT = a.mf / 32;
    const int key = 32 * kt + l32;
    const bool live = key < a.k;
    const long img_plane = (long)a.BH * a.kp * D;
    const long ds_plane = (long)a.BH * a.mf * D;
    constexpr int P = BwdKeyLds<D>::pitch;
    unsigned char* tw = lds + wave * 3 * BwdKeyLds<D>::tile;       // omega | dS hi | dS lo
    const int s16 = lane & 15;
    const int tr_off = (4 * half + (s16 >> 2)) * P + 2 * (16 * ((lane >> 4) & 1) + 4 * (s16 & 3));

    // The tile's rows of K' and V' (32 x D fp32 each, contiguous in ctx) are fetched once per workgroup
    // with whole-line loads into LDS (rows past k as zeros); every wavefront then takes this lane's key
    // out of it (8 consecutive coordinates per step, split into bf16 terms: B operands) and the K'
    // entries its part of the epilogue needs.  The area is reused by the feature tiles below.
    constexpr int SP = D * 4 + 16;                  // staging row pitch: 16-byte reads down a column of rows
    {
        constexpr int CPRF = D / 4;                 // 16-byte chunks per fp32 row
        for (int c = threadIdx.x; c < 32 * CPRF; c += 256) {
            const int row = c / CPRF, q = c % CPRF;
            const int r = 32 * kt + row;
            float4 x = {0.f, 0.f, 0.f, 0.f}, y = {0.f, 0.f, 0.f, 0.f};
            if (r < a.k) {
                x = *(const float4*)(a.Kp + ((long)bh * a.k + r) * D + 4 * q);
                y = *(const float4*)(a.Vp + ((long)bh * a.k + r) * D + 4 * q);
            }
            *(float4*)(lds + row * SP + 16 * q) = x;
            *(float4*)(lds + 32 * SP + row * SP + 16 * q) = y;
        }
    }
    __syncthreads();
    uint4 kb[3][KS], vb[2][KS];
    float nrm = 0.f;
    float kpr[TT][4];                               // K'[32*kt + 8*wave + 4*half + i][32*tt + l32]
    {
        const unsigned char* kg = lds + l32 * SP + 32 * half;
        const unsigned char* vg = kg + 32 * SP;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            float kv[8], vv[8];
            *(float4*)&kv[0] = *(const float4*)(kg + 64 * s);
            *(float4*)&kv[4] = *(const float4*)(kg + 64 * s + 16);
            *(float4*)&vv[0] = *(const float4*)(vg + 64 * s);
            *(float4*)&vv[4] = *(const float4*)(vg + 64 * s + 16);
            uint32_t kh[4], km[4], kl[4], vh[4], vl[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                split3_pair(kv[2 * e], kv[2 * e + 1], kh[e], km[e], kl[e]);
                nrm = fmaf(kv[2 * e], kv[2 * e], nrm);
                nrm = fmaf(kv[2 * e + 1], kv[2 * e + 1], nrm);
                split2_pair(vv[2 * e], vv[2 * e + 1], vh[e], vl[e]);
            }
            kb[0][s] = make_uint4(kh[0], kh[1], kh[2], kh[3]);
            kb[1][s] = make_uint4(km[0], km[1], km[2], km[3]);
            kb[2][s] = make_uint4(kl[0], kl[1], kl[2], kl[3]);
            vb[0][s] = make_uint4(vh[0], vh[1], vh[2], vh[3]);
            vb[1][s] = make_uint4(vl[0], vl[1], vl[2], vl[3]);
        }
        nrm = half_sum(nrm);
        nrm = live ? 0.5f * nrm : INFINITY;       // padding keys: exponent -inf, PhiK = 0
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                kpr[tt][i] = *(const float*)(lds + (8 * wave + 4 * half + i) * SP + 4 * (32 * tt + l32));
    }
    __syncthreads();                              // the staging area becomes the wavefronts' tile areas

    floatx16 accV[TT], accK[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) { accV[t] = zero16(); accK[t] = zero16(); }
    float rs = 0.f;
    // A feature of the padding (ragged last tile) has dS = 0 and dz = 0 by construction; it takes the
    // omega row and the shift of the last real feature, so that its PhiK is finite and multiplies those 0.
    const float* cg = a.c + (long)bh * a.mr;
    const float* zg = a.dz + (long)bh * a.mf + 4 * half;

    for (int ft = wave; ft < FT; ft += 4) {
        float4 cv4[4], zv4[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int f0 = 32 * ft + 8 * q + 4 * half, last = a.mr - 1;     // ctx rows are mr long: scalar loads
            cv4[q].x = cg[f0 < last ? f0 : last];
            cv4[q].y = cg[f0 + 1 < last ? f0 + 1 : last];
            cv4[q].z = cg[f0 + 2 < last ? f0 + 2 : last];
            cv4[q].w = cg[f0 + 3 < last ? f0 + 3 : last];
            zv4[q] = *(const float4*)(zg + 32 * ft + 8 * q);
        }
        {   // this feature tile's rows of omega and dS, row-major, into the wavefront's LDS area
            constexpr int CPR = D / 8, LPT = 32 * CPR / 64;
            const uint16_t* ob = a.omega + (long)(bh % a.H) * a.omega_head_stride + (long)(32 * ft) * D;
            const uint16_t* sb = a.dSimg + ((long)bh * a.mf + 32 * ft) * D;
#pragma unroll
            for (int u = 0; u < LPT; ++u) {
                const int chunk = lane + 64 * u, row = chunk / CPR, c = chunk % CPR;
                const uint4 x0 = ld16(ob + (32 * ft + row < a.mr ? row : a.mr - 1 - 32 * ft) * D + 8 * c);
                const uint4 x1 = ld16(sb + row * D + 8 * c);
                const uint4 x2 = ld16(sb + ds_plane + row * D + 8 * c);
                unsigned char* dst = tw + row * P + 16 * c;
                *(uint4*)dst = x0;
                *(uint4*)(dst + BwdKeyLds<D>::tile) = x1;
                *(uint4*)(dst + 2 * BwdKeyLds<D>::tile) = x2;
            }
        }
        // e^T tile (features x keys) and dPhiK^T tile; element g <-> feature 32*ft + 8*(g/4) + 4*half + g%4.
        // The A operands (this lane's feature row, 8 coordinates per step) come out of the tiles just
        // copied; c and dz of the tile were requested together with them.
        floatx16 e = zero16(), dp;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            dp[4 * q] = zv4[q].x; dp[4 * q + 1] = zv4[q].y; dp[4 * q + 2] = zv4[q].z; dp[4 * q + 3] = zv4[q].w;
        }
        const unsigned char* arow = tw + l32 * P + 16 * half;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint4 wa = *(const uint4*)(arow + 32 * s);
            e = mfma32(wa, kb[0][s], e);
            e = mfma32(wa, kb[1][s], e);
            e = mfma32(wa, kb[2][s], e);
            const uint4 dh = *(const uint4*)(arow + BwdKeyLds<D>::tile + 32 * s);
            const uint4 dl = *(const uint4*)(arow + 2 * BwdKeyLds<D>::tile + 32 * s);
            dp = mfma32(dh, vb[0][s], dp);
            dp = mfma32(dl, vb[0][s], dp);
            dp = mfma32(dh, vb[1][s], dp);
        }
        uint32_t ph[8], pl[8], uh[8], ul[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float cc[4] = {cv4[q].x, cv4[q].y, cv4[q].z, cv4[q].w};
            float phi[4], du[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                phi[i] = fast_exp2((e[4 * q + i] - nrm - cc[i]) * LOG2E);
                du[i] = dp[4 * q + i] * phi[i];
                rs += du[i];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                split2_pair(phi[2 * i], phi[2 * i + 1], ph[2 * q + i], pl[2 * q + i]);
                split2_pair(du[2 * i], du[2 * i + 1], uh[2 * q + i], ul[2 * q + i]);
            }
        }
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
            const uint4 pah = {ph[4 * sp], ph[4 * sp + 1], ph[4 * sp + 2], ph[4 * sp + 3]};
            const uint4 pal = {pl[4 * sp], pl[4 * sp + 1], pl[4 * sp + 2], pl[4 * sp + 3]};
            const uint4 uah = {uh[4 * sp], uh[4 * sp + 1], uh[4 * sp + 2], uh[4 * sp + 3]};
            const uint4 ual = {ul[4 * sp], ul[4 * sp + 1], ul[4 * sp + 2], ul[4 * sp + 3]};
            // B operands: column t = 32*tt + l32 of features 32*ft + 16*sp + 4*half + {0..3, 8..11}
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const unsigned char* bp = tw + tr_off + (16 * sp) * P + 64 * tt;
                const uint2 w0 = lds_read_tr16(bp), w1 = lds_read_tr16(bp + 8 * P);
                const uint2 h0 = lds_read_tr16(bp + BwdKeyLds<D>::tile), h1 = lds_read_tr16(bp + BwdKeyLds<D>::tile + 8 * P);
                const uint2 l0 = lds_read_tr16(bp + 2 * BwdKeyLds<D>::tile), l1 = lds_read_tr16(bp + 2 * BwdKeyLds<D>::tile + 8 * P);
                const uint4 bw4 = {w0.x, w0.y, w1.x, w1.y};
                const uint4 bh4 = {h0.x, h0.y, h1.x, h1.y};
                const uint4 bl4 = {l0.x, l0.y, l1.x, l1.y};
                accV[tt] = mfma32(pah, bh4, accV[tt]);
                accV[tt] = mfma32(pal, bh4, accV[tt]);
                accV[tt] = mfma32(pah, bl4, accV[tt]);
                accK[tt] = mfma32(uah, bw4, accK[tt]);
                accK[tt] = mfma32(ual, bw4, accK[tt]);
            }
        }
    }
    rs = half_sum(rs);

    // add the four wavefronts' partial results: slot w = [dV' | dK'][tt][g][lane], then rs[lane]
    __syncthreads();                    // the slots reuse the tile area
    float* slots = (float*)lds;
    constexpr int SLOT = 2 * TT * 16 * 64 + 64;
    {
        float* my = slots + wave * SLOT;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                my[(tt * 16 + g) * 64 + lane] = accV[tt][g];
                my[((TT + tt) * 16 + g) * 64 + lane] = accK[tt][g];
            }
        my[2 * TT * 16 * 64 + lane] = rs;
    }
    __syncthreads();

    // wavefront w finishes key group q = w: rows (keys) 32*kt + 8*w + 4*half + {0..3}, column t = 32*tt + l32
    uint16_t* imgK = a.img;
    uint16_t* imgV = a.img + img_plane;
    uint16_t* imgTK = a.imgT;
    uint16_t* imgTV = a.imgT + img_plane;
    const int q = wave;
    const int r0 = 32 * kt + 8 * q + 4 * half;
    float rsq[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int src = 8 * q + 4 * half + i;                // lane that holds this key's row sum
        rsq[i] = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) rsq[i] += slots[w * SLOT + 2 * TT * 16 * 64 + src];
    }
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int t = 32 * tt + l32;
        float dk[4], dv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float sv = 0.f, sk = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                sv += slots[w * SLOT + (tt * 16 + 4 * q + i) * 64 + lane];
                sk += slots[w * SLOT + ((TT + tt) * 16 + 4 * q + i) * 64 + lane];
            }
            dk[i] = sk - rsq[i] * kpr[tt][i];
            dv[i] = sv;
        }
        uint2 pk, pv;
        pk.x = pack_bf16(dk[0], dk[1]); pk.y = pack_bf16(dk[2], dk[3]);
        pv.x = pack_bf16(dv[0], dv[1]); pv.y = pack_bf16(dv[2], dv[3]);
        const uint32_t pkw[2] = {pk.x, pk.y}, pvw[2] = {pv.x, pv.y};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const long io = ((long)bh * a.kp + r0 + i) * D + t;
            imgK[io] = (uint16_t)(pkw[i >> 1] >> (16 * (i & 1)));
            imgV[io] = (uint16_t)(pvw[i >> 1] >> (16 * (i & 1)));
        }
        *(uint2*)(imgTK + ((long)bh * D + t) * a.kp + r0) = pk;
        *(uint2*)(imgTV + ((long)bh * D + t) * a.kp + r0) = pv;
    }
}

// dE, dF (k x n, bf16) = sum over splits of the tile-ordered fp32 partials of the dE/dF GEMM (layout in
// flurka_gemm.h).  One thread = four consecutive rows (the four floats of one 16-byte element) of two
// adjacent columns (two adjacent elements): 32 contiguous bytes per split.  blockIdx.y: dE or dF.
struct SumSplitsArgs {
    uint16_t* dst[2];
    const float* part;
    int k, n, splits, tilesM, tilesN;
};

__global__ __launch_bounds__(256) void sum_splits_bf16_kernel(SumSplitsArgs a) {
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const int half_n = a.n / 2;
    const int c = 2 * (int)(gid % half_n);
    const int r0 = 4 * (int)(gid / half_n);
    if (r0 >= a.k) return;
    const int which = blockIdx.y;
    const int tm = r0 / GBM, tn = c / GBN;
    const int eo = partial_elem_offset(r0 % GBM, c % GBN);
    float4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < a.splits; ++s) {
        const float* tp = a.part + partial_tile_index(which, s, tn, tm, a.splits, a.tilesN, a.tilesM) * G_TILE_ELEMS + eo;
        const float4 x = *(const float4*)tp, y = *(const float4*)(tp + 4);
        s0.x += x.x; s0.y += x.y; s0.z += x.z; s0.w += x.w;
        s1.x += y.x; s1.y += y.y; s1.z += y.z; s1.w += y.w;
    }
    uint16_t* o = a.dst[which] + (long)r0 * a.n + c;
    const float v0[4] = {s0.x, s0.y, s0.z, s0.w}, v1[4] = {s1.x, s1.y, s1.z, s1.w};
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (r0 + e < a.k) *(uint32_t*)(o + (long)e * a.n) = pack_bf16(v0[e], v1[e]);
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
// bwd_query_x keeps all its operand images in LDS where they fit; at d = 128 the lo terms of S/z go
// through a two-slot ring otherwise (see BwdXLds)
static bool bwd_x_ring(const Problem& p) { return p.d == 128 && BwdXLds<128>::total(p.mfp) > 160 * 1024; }
static int bwd_x_lds_bytes(const Problem& p) {
    if (p.d == 64) return BwdXLds<64>::total(p.mfp);
    return bwd_x_ring(p) ? BwdXLds<128, true>::total(p.mfp) : BwdXLds<128>::total(p.mfp);
}

bool fast_bwd_supported(const Problem& p) {
    if (!p.bf16) return false;
    if (p.d != 64 && p.d != 128) return false;
    if (p.n % 32 != 0) return false;                         // whole 32-row query tiles
    if (!p.elu && bwd_x_lds_bytes(p) > 160 * 1024) return false;
    // 32-bit byte offsets inside the gradient GEMMs' buffer descriptors
    if ((size_t)p.BH * p.n * p.d * 2 >= ((size_t)1 << 31)) return false;
    if (((size_t)p.k + GBM) * (size_t)p.n * 2 >= ((size_t)1 << 31)) return false;
    // ... and inside the bf16 images of dK', dV' (k may exceed n): BH*d rows of kp slots each, plus the rows
    // of a last tile that reach past the end
    const size_t kp = ((size_t)p.k + 63) / 64 * 64;
    if (((size_t)p.BH * p.d + GBM) * kp * 2 >= ((size_t)1 << 31)) return false;
    return true;
}

struct GradEPlan {
    int tilesM, tilesN, total_steps, splits, steps_per_split;
    int resident;          // workgroups of the launch dE/dF share with dK/dV
    PairPlan pair;
};

// dE/dF (few items with a reduction over all B*H*d/64 steps) share their launch with dK/dV (many items of
// kp/64 steps).  Unsplit, the long items are the critical path whenever there are fewer of them than
// compute units (64 at the headline size: 89 us, the short items done after 46); split s ways they
// finish sooner, their workgroups go on with short items, and a second pass sums the s partial results.
// The split that the cost model (plan_pair, plus the traffic of the second pass) expects to finish first
// wins.
static GradEPlan grad_e_plan(const Problem& p) {
    GradEPlan q;
    q.tilesM = (p.k + GBM - 1) / GBM;
    q.tilesN = (p.n + GBN - 1) / GBN;
    q.total_steps = p.BH * p.d / GBK;
    q.resident = chip_cus() / 8 * 8;
    const int kp = (p.k + 63) / 64 * 64;
    const int items_b = 8 * ((p.BH * p.d + GBM - 1) / GBM) * ((q.tilesN * 2 + 7) / 8);
    const int steps_b = kp / GBK;
    double best = -1.0;
    for (int want = 1; want <= 8; ++want) {
        if (want > q.total_steps) break;
        const int sps = (q.total_steps + want - 1) / want;
        const int splits = (q.total_steps + sps - 1) / sps;
        if (splits != want) continue;
        const int items_a = 8 * q.tilesM * ((splits * q.tilesN * 2 + 7) / 8);
        double t = 0.0;
        const PairPlan pl = plan_pair(items_a, sps, items_b, steps_b, q.resident, &t);
        if (splits > 1) {
            // second pass: reads the fp32 partials, writes bf16; about 4 TB/s plus a launch
            const double bytes = 2.0 * q.tilesM * q.tilesN * G_TILE_ELEMS * 4.0 * splits + 4.0 * p.k * (double)p.n;
            t += 4.0 + bytes / 4.0e6;
        }
        if (best < 0.0 || t < best) {
            best = t;
            q.splits = splits; q.steps_per_split = sps; q.pair = pl;
        }
    }
    return q;
}

struct BwdYPlan { int FT, NW, R, tiles_per_range; };

static BwdYPlan bwd_y_plan(const Problem& p) {
    BwdYPlan q;
    q.FT = p.mfp / 32;
    q.NW = q.FT > 4 ? 8 : 4;                      // wavefronts (= feature tiles) per workgroup
    const int QT = p.n / 32;
    const int FG = (q.FT + q.NW - 1) / q.NW;
    // one round of workgroups: the chip holds one 8-wavefront or two 4-wavefront workgroups per
    // compute unit; ranges are whole staged blocks of query tiles
    const int slots = 2 * chip_cus();
    int R = slots / (p.BH * FG);
    if (R > QT / Y_ST) R = QT / Y_ST;
    if (R < 1) R = 1;
    q.tiles_per_range = ((QT + R - 1) / R + Y_ST - 1) / Y_ST * Y_ST;
    q.R = (QT + q.tiles_per_range - 1) / q.tiles_per_range;
    return q;
}

struct FastBwdWs {
    size_t delta, lam2, dSpart, dzpart, dSimg, dz, img, imgT, epart, total;
    int kp;      // k rounded up to whole 64-slot reduction steps of the gradient GEMMs
};

static FastBwdWs fast_bwd_ws_layout(const Problem& p) {
    FastBwdWs W{};
    const BwdYPlan y = bwd_y_plan(p);
    const size_t BH = (size_t)p.BH;
    size_t o = 0;
    W.delta = o;  o += round_up(BH * p.n * 4, 256);
    W.lam2 = o;   o += round_up(BH * p.n * 4, 256);
    W.dSpart = o; o += round_up(BH * y.R * p.mfp * p.d * 4, 256);
    W.dzpart = o; o += round_up(BH * y.R * p.mfp * 4, 256);
    W.dSimg = o;  o += round_up(2 * BH * p.mfp * p.d * 2, 256);
    W.dz = o;     o += round_up(BH * p.mfp * 4, 256);
    W.kp = (p.k + 63) / 64 * 64;
    const GradEPlan e = grad_e_plan(p);
    W.img = o;    o += round_up(2 * BH * W.kp * p.d * 2, 256);        // dK' then dV'
    W.imgT = o;   o += round_up(2 * BH * W.kp * p.d * 2, 256);
    // tile-ordered dE, dF partials (none when the reduction is not split)
    W.epart = o;  o += e.splits == 1 ? 0 : round_up((size_t)2 * e.splits * e.tilesM * e.tilesN * G_TILE_ELEMS * 4, 256);
    W.total = o;
    return W;
}

// elu1: the key side runs on the generic kernels, whose workspace comes first
struct EluBwdWs {
    size_t delta, dinv, dSpart, dzpart, img, imgT, epart, total;
    int kp;
};

static EluBwdWs elu_bwd_ws_layout(const Problem& p) {
    EluBwdWs W{};
    const BwdYPlan y = bwd_y_plan(p);
    const GradEPlan e = grad_e_plan(p);
    const size_t BH = (size_t)p.BH;
    size_t o = round_up(generic_ws_layout(p, 1).total * sizeof(float), 256);
    W.delta = o;  o += round_up(BH * p.n * 4, 256);
    W.dinv = o;   o += round_up(BH * p.n * 4, 256);
    W.dSpart = o; o += round_up(BH * y.R * p.mfp * p.d * 4, 256);
    W.dzpart = o; o += round_up(BH * y.R * p.mfp * 4, 256);
    W.kp = (p.k + 63) / 64 * 64;
    W.img = o;    o += round_up(2 * BH * W.kp * p.d * 2, 256);
    W.imgT = o;   o += round_up(2 * BH * W.kp * p.d * 2, 256);
    W.epart = o;  o += e.splits == 1 ? 0 : round_up((size_t)2 * e.splits * e.tilesM * e.tilesN * G_TILE_ELEMS * 4, 256);
    W.total = o;
    return W;
}

size_t fast_bwd_ws_bytes(const Problem& p) { return p.elu ? elu_bwd_ws_layout(p).total : fast_bwd_ws_layout(p).total; }

template <int D, int NW, bool ELU>
static flurka_status launch_bwd_y_impl(const BwdYArgs& ya, unsigned grid, hipStream_t s) {
    auto kern = bwd_query_y_kernel<D, NW, ELU>;
    constexpr int ldsb = BwdYLds<D, ELU>::total;
    KernelFacts facts;
    if (!kernel_facts((const void*)kern, NW * 64, ldsb, &facts)) return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), ldsb, s, ya);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

static flurka_status launch_bwd_y(const Problem& p, const BwdYArgs& ya, const BwdYPlan& y, hipStream_t s) {
    const unsigned grid = (unsigned)((long)p.BH * y.R * ((y.FT + y.NW - 1) / y.NW));
    if (p.elu) {        // features = the d coordinates: 2 or 4 feature tiles
        return p.d == 64 ? launch_bwd_y_impl<64, 4, true>(ya, grid, s) : launch_bwd_y_impl<128, 4, true>(ya, grid, s);
    }
    if (p.d == 64) return y.NW == 8 ? launch_bwd_y_impl<64, 8, false>(ya, grid, s) : launch_bwd_y_impl<64, 4, false>(ya, grid, s);
    return y.NW == 8 ? launch_bwd_y_impl<128, 8, false>(ya, grid, s) : launch_bwd_y_impl<128, 4, false>(ya, grid, s);
}

template <int D, bool RING>
static flurka_status launch_bwd_x(const BwdXArgs& xa, int ldsb, hipStream_t s) {
    auto kern = bwd_query_x_kernel<D, RING>;
    constexpr int threads = BwdXLds<D, RING>::nw * 64;
    const int grid = resident_grid((const void*)kern, threads, ldsb, xa.total_tiles);
    if (grid < 1) return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), ldsb, s, xa);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

// The four sequence-length GEMMs from the bf16 images of dK', dV': img (2 x BH x kp x d) and imgT
// (2 x BH*d x kp); `part` holds the split partials of dE, dF.  dE/dF (few long items) and dK/dV (many
// short items) run side by side in one launch.
template <int D>
static flurka_status grad_gemms_d(const Problem& p, const BwdArgs& a, const uint16_t* img, const uint16_t* imgT,
                                  int kp, float* part, hipStream_t s) {
    const size_t img_elems = (size_t)p.BH * kp * p.d;
    const GradEPlan e = grad_e_plan(p);
    GemmParams gx{};       // dK = E^T dK', dV = F^T dV'
    gx.A[0] = imgT; gx.A[1] = imgT + img_elems;
    gx.B[0] = (const uint16_t*)a.E; gx.B[1] = (const uint16_t*)a.F;
    gx.C[0] = a.dK; gx.C[1] = a.dV;
    gx.n = p.n; gx.d = p.d; gx.k = p.k; gx.BH = p.BH; gx.kp = kp;
    gx.tilesM = (p.BH * p.d + GBM - 1) / GBM; gx.tilesN = (p.n + GBN - 1) / GBN;
    gx.splits = 1; gx.total_steps = kp / GBK; gx.steps_per_split = gx.total_steps;
    GemmParams ge{};       // dE = sum_bh dK' K^T, dF = sum_bh dV' V^T
    ge.A[0] = img; ge.A[1] = img + img_elems;
    ge.B[0] = (const uint16_t*)a.K; ge.B[1] = (const uint16_t*)a.V;
    ge.n = p.n; ge.d = p.d; ge.k = p.k; ge.BH = p.BH; ge.kp = kp;
    ge.tilesM = e.tilesM; ge.tilesN = e.tilesN; ge.splits = e.splits;
    ge.total_steps = e.total_steps; ge.steps_per_split = e.steps_per_split;
    flurka_status st;
    {
        StageScope sc(s, STAGE_K_GRAD_PAIR);
        if (e.splits == 1) {
            // enough tiles to fill the chip without splitting the reduction: results leave as bf16
            ge.C[0] = a.dE; ge.C[1] = a.dF;
            st = launch_gemm_mfma_pair<GradEPolicy<D, true>, GradXPolicy<D>>(ge, gx, e.pair, e.resident, s);
        } else {
            ge.C[0] = part; ge.C[1] = nullptr;
            st = launch_gemm_mfma_pair<GradEPolicy<D, false>, GradXPolicy<D>>(ge, gx, e.pair, e.resident, s);
        }
        if (st != FLURKA_OK) return st;
    }
    if (e.splits > 1) {
        StageScope sc(s, STAGE_K_SUM_SPLITS);
        SumSplitsArgs sa{};
        sa.dst[0] = (uint16_t*)a.dE; sa.dst[1] = (uint16_t*)a.dF; sa.part = part;
        sa.k = p.k; sa.n = p.n; sa.splits = e.splits; sa.tilesM = e.tilesM; sa.tilesN = e.tilesN;
        const long threads = (long)((p.k + 3) / 4) * (p.n / 2);
        hipLaunchKernelGGL(sum_splits_bf16_kernel, dim3((unsigned)((threads + 255) / 256), 2), dim3(256), 0, s, sa);
        FLURKA_CHECK_LAUNCH();
    }
    return FLURKA_OK;
}

static flurka_status grad_gemms(const Problem& p, const BwdArgs& a, const uint16_t* img, const uint16_t* imgT,
                                int kp, float* part, hipStream_t s) {
    return p.d == 64 ? grad_gemms_d<64>(p, a, img, imgT, kp, part, s) : grad_gemms_d<128>(p, a, img, imgT, kp, part, s);
}

static flurka_status fast_backward_elu(const Problem& p, const BwdArgs& a, hipStream_t s);

flurka_status fast_backward(const Problem& p, const BwdArgs& a, hipStream_t s) {
    if (p.elu) return fast_backward_elu(p, a, s);
    const CtxLayout L = ctx_layout(p);
    const FastBwdWs W = fast_bwd_ws_layout(p);
    const BwdYPlan y = bwd_y_plan(p);
    unsigned char* wsb = (unsigned char*)a.ws;
    const long omega_stride = p.omega_per_head ? (long)p.m * p.d : 0;
    flurka_status st;
    {
        BwdXArgs xa{};
        xa.Q = (const uint16_t*)a.Q; xa.G = (const uint16_t*)a.dOut; xa.omega = (const uint16_t*)a.omega;
        xa.O = (const uint16_t*)a.out;
        xa.S = a.ctx + L.S; xa.z = a.ctx + L.z; xa.c = a.ctx + L.c;
        xa.dQ = (uint16_t*)a.dQ; xa.lse = a.ctx + L.lse; xa.delta = (float*)(wsb + W.delta);
        xa.lam2 = (float*)(wsb + W.lam2);
        xa.n = p.n; xa.H = p.H; xa.mf = p.mfp; xa.mr = p.mf; xa.omega_head_stride = omega_stride;
        xa.tiles_per_head = (p.n + 31) / 32;
        xa.total_tiles = (long)p.BH * xa.tiles_per_head;
        const int ldsb = bwd_x_lds_bytes(p);
        stage_begin(s);
        st = p.d == 64 ? launch_bwd_x<64, false>(xa, ldsb, s)
             : bwd_x_ring(p) ? launch_bwd_x<128, true>(xa, ldsb, s) : launch_bwd_x<128, false>(xa, ldsb, s);
        if (st != FLURKA_OK) return st;
        stage_end(s, STAGE_K_BWD_X);

        BwdYArgs ya{};
        ya.Q = xa.Q; ya.G = xa.G; ya.omega = xa.omega; ya.c = a.ctx + L.c;
        ya.lse = xa.lam2; ya.delta = xa.delta;
        ya.dSpart = (float*)(wsb + W.dSpart); ya.dzpart = (float*)(wsb + W.dzpart);
        ya.omega_head_stride = omega_stride;
        ya.BH = p.BH; ya.H = p.H; ya.n = p.n; ya.mf = p.mfp; ya.mr = p.mf; ya.FT = y.FT; ya.R = y.R;
        ya.tiles_per_range = y.tiles_per_range;
        stage_begin(s);
        if ((st = launch_bwd_y(p, ya, y, s)) != FLURKA_OK) return st;
        FLURKA_CHECK_LAUNCH();
        stage_end(s, STAGE_K_BWD_Y);
    }
    uint16_t* img = (uint16_t*)(wsb + W.img);
    uint16_t* imgT = (uint16_t*)(wsb + W.imgT);
    {
        stage_begin(s);
        const long mtotal = (long)p.BH * (p.mfp / 2) * p.d;
        hipLaunchKernelGGL(bwd_merge_kernel, grid1d(mtotal, 256), dim3(256), 0, s, (uint16_t*)(wsb + W.dSimg),
                           (float*)nullptr, (float*)(wsb + W.dz), (const float*)(wsb + W.dSpart),
                           (const float*)(wsb + W.dzpart), y.R, p.mfp, p.d, mtotal);
        FLURKA_CHECK_LAUNCH();
        stage_end(s, STAGE_K_BWD_MERGE);
        StageScope sc(s, STAGE_K_BWD_KEY);
        BwdKeyArgs ka{};
        ka.Kp = a.ctx + L.Kp; ka.Vp = a.ctx + L.Vp; ka.c = a.ctx + L.c;
        ka.omega = (const uint16_t*)a.omega;
        ka.dSimg = (const uint16_t*)(wsb + W.dSimg);
        ka.dz = (const float*)(wsb + W.dz);
        ka.img = img; ka.imgT = imgT;
        ka.omega_head_stride = omega_stride;
        ka.BH = p.BH; ka.H = p.H; ka.k = p.k; ka.kp = W.kp; ka.mf = p.mfp; ka.mr = p.mf;
        const unsigned kgrid = (unsigned)((p.BH + 7) / 8 * 8 * (W.kp / 32));
        const int klds = p.d == 64 ? BwdKeyLds<64>::total : BwdKeyLds<128>::total;
        const void* kk = p.d == 64 ? (const void*)bwd_key_kernel<64> : (const void*)bwd_key_kernel<128>;
        KernelFacts facts;
        if (!kernel_facts(kk, 256, klds, &facts)) return FLURKA_ERR_LAUNCH;
        if (p.d == 64) hipLaunchKernelGGL(bwd_key_kernel<64>, dim3(kgrid), dim3(256), klds, s, ka);
        else           hipLaunchKernelGGL(bwd_key_kernel<128>, dim3(kgrid), dim3(256), klds, s, ka);
        FLURKA_CHECK_LAUNCH();
    }
    return grad_gemms(p, a, img, imgT, W.kp, (float*)(wsb + W.epart), s);
}

// elu1: dQ, dS, dz on MFMA kernels of their own; the small key side on the generic kernels (0.05 ms at
// k = 256); the four sequence-length GEMMs as for the random-feature map.
template <int D>
static flurka_status launch_bwd_x_elu(const BwdXEluArgs& xa, hipStream_t s) {
    auto kern = bwd_query_x_elu_kernel<D>;
    constexpr int ldsb = BwdXEluLds<D>::total;
    const int grid = resident_grid((const void*)kern, 512, ldsb, xa.total_tiles);
    if (grid < 1) return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), ldsb, s, xa);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

// ---------------------------------------------------------------------------
// elu1 key side in one kernel (features = the d coordinates, so dS is d x d per head and everything a
// key needs fits one workgroup): Phi = elu(K') + 1,
//     dPhi_rj = sum_t V'_rt dS_jt + dz_j,   dK'_rj = dPhi_rj phi'(K'_rj),   dV'_rt = sum_j Phi_rj dS_jt,
// all in fp32, results written straight as the bf16 operand images of the gradient GEMMs (img
// (BH, kp, d) with zero rows past k, imgT (BH * d, kp); dV' follows dK' in both).  One workgroup per
// (head, 32 keys); thread = (key, 8 columns).  The work is 4 d^2 flop per key: what matters is that it
// is one launch.
// ---------------------------------------------------------------------------
template <int D>
struct BwdKeyEluLds {
    static constexpr int P = D + 1;                                        // padded row, floats
    static constexpr int total = (D * P + 3 * 32 * P + D) * 4;            // dS, K', V', Phi tiles, dz
};

template <int D>
__global__ __launch_bounds__(256) void bwd_key_elu_fused_kernel(const float* Kp, const float* Vp, const float* dS,
                                                                const float* dz, uint16_t* img, uint16_t* imgT,
                                                                int BH, int k, int kp) {
    extern __shared__ __attribute__((aligned(16))) float elu_key_lds[];
    constexpr int P = BwdKeyEluLds<D>::P;
    float* sdS = elu_key_lds;                   // [D][P]: dS[j][t]
    float* sK = sdS + D * P;           // [32][P]: K' tile, later dK'
    float* sV = sK + 32 * P;           // [32][P]: V' tile, later dV'
    float* sPhi = sV + 32 * P;         // [32][P]
    float* sdz = sPhi + 32 * P;        // [D]
    const int tid = threadIdx.x;
    const int KT = kp / 32;
    const int kt = (int)(blockIdx.x % KT);
    const long bh = blockIdx.x / KT;
    for (int i = tid; i < D * D; i += 256) sdS[(i / D) * P + i % D] = dS[bh * D * D + i];
    for (int i = tid; i < D; i += 256) sdz[i] = dz[bh * D + i];
    for (int i = tid; i < 32 * D; i += 256) {
        const int r = i / D, t = i % D, key = 32 * kt + r;
        const float kv = key < k ? Kp[(bh * k + key) * D + t] : 0.f;
        sK[r * P + t] = kv;
        sV[r * P + t] = key < k ? Vp[(bh * k + key) * D + t] : 0.f;
        sPhi[r * P + t] = elu1_of(kv);
    }
    __syncthreads();
    const int r = tid >> 3, g = tid & 7;
    const bool live = 32 * kt + r < k;
    float rk[D / 8], rv[D / 8];
#pragma unroll
    for (int i = 0; i < D / 8; ++i) { rk[i] = sdz[g + 8 * i]; rv[i] = 0.f; }
    for (int t = 0; t < D; ++t) {
        const float v = sV[r * P + t], ph = sPhi[r * P + t];
#pragma unroll
        for (int i = 0; i < D / 8; ++i) {
            rk[i] = fmaf(v, sdS[(g + 8 * i) * P + t], rk[i]);        // dPhi_rc, c = g + 8i
            rv[i] = fmaf(ph, sdS[t * P + g + 8 * i], rv[i]);         // dV'_rc
        }
    }
#pragma unroll
    for (int i = 0; i < D / 8; ++i) {
        const float x = sK[r * P + g + 8 * i];
        rk[i] = live ? rk[i] * (x > 0.f ? 1.f : __expf(x)) : 0.f;
        rv[i] = live ? rv[i] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < D / 8; ++i) {
        sK[r * P + g + 8 * i] = rk[i];
        sV[r * P + g + 8 * i] = rv[i];
    }
    __syncthreads();
    const long per_tensor = (long)BH * kp * D;
    for (int i = tid; i < 32 * D; i += 256) {             // rows of the images: D consecutive columns
        const int rr = i / D, c = i % D;
        const long o = (bh * kp + 32 * kt + rr) * D + c;
        img[o] = (uint16_t)pack_bf16(sK[rr * P + c], 0.f);
        img[per_tensor + o] = (uint16_t)pack_bf16(sV[rr * P + c], 0.f);
    }
    for (int i = tid; i < 32 * D; i += 256) {             // transposed images: 32 consecutive keys
        const int c = i / 32, rr = i % 32;
        const long o = (bh * D + c) * kp + 32 * kt + rr;
        imgT[o] = (uint16_t)pack_bf16(sK[rr * P + c], 0.f);
        imgT[per_tensor + o] = (uint16_t)pack_bf16(sV[rr * P + c], 0.f);
    }
}

template <int D>
static flurka_status launch_bwd_key_elu(const Problem& p, const float* Kp, const float* Vp, const float* dS,
                                        const float* dz, uint16_t* img, uint16_t* imgT, int kp, hipStream_t s) {
    auto kern = bwd_key_elu_fused_kernel<D>;
    constexpr int ldsb = BwdKeyEluLds<D>::total;
    KernelFacts facts;
    if (!kernel_facts((const void*)kern, 256, ldsb, &facts)) return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.BH * (kp / 32))), dim3(256), ldsb, s, Kp, Vp, dS, dz, img, imgT, p.BH,
                       p.k, kp);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

static flurka_status fast_backward_elu(const Problem& p, const BwdArgs& a, hipStream_t s) {
    const CtxLayout L = ctx_layout(p);
    const GenericWs GW = generic_ws_layout(p, 1);
    const EluBwdWs W = elu_bwd_ws_layout(p);
    const BwdYPlan y = bwd_y_plan(p);
    unsigned char* wsb = (unsigned char*)a.ws;
    flurka_status st;
    {
        BwdXEluArgs xa{};
        xa.Q = (const uint16_t*)a.Q; xa.G = (const uint16_t*)a.dOut;
        xa.S = a.ctx + L.S; xa.z = a.ctx + L.z;
        xa.dQ = (uint16_t*)a.dQ; xa.delta = (float*)(wsb + W.delta); xa.dinv = (float*)(wsb + W.dinv);
        xa.n = p.n; xa.tiles_per_head = (p.n + 31) / 32;
        xa.total_tiles = (long)p.BH * xa.tiles_per_head;
        stage_begin(s);
        st = p.d == 64 ? launch_bwd_x_elu<64>(xa, s) : launch_bwd_x_elu<128>(xa, s);
        if (st != FLURKA_OK) return st;
        stage_end(s, STAGE_K_BWD_X);

        BwdYArgs ya{};
        ya.Q = xa.Q; ya.G = xa.G; ya.lse = xa.dinv; ya.delta = xa.delta;
        ya.dSpart = (float*)(wsb + W.dSpart); ya.dzpart = (float*)(wsb + W.dzpart);
        ya.BH = p.BH; ya.H = p.H; ya.n = p.n; ya.mf = p.mfp; ya.mr = p.mf; ya.FT = y.FT; ya.R = y.R;
        ya.tiles_per_range = y.tiles_per_range;
        stage_begin(s);
        if ((st = launch_bwd_y(p, ya, y, s)) != FLURKA_OK) return st;
        stage_end(s, STAGE_K_BWD_Y);

        stage_begin(s);
        const long mtotal = (long)p.BH * (p.mfp / 2) * p.d;
        hipLaunchKernelGGL(bwd_merge_kernel, grid1d(mtotal, 256), dim3(256), 0, s, (uint16_t*)nullptr,
                           a.ws + GW.dS, a.ws + GW.dz, (const float*)(wsb + W.dSpart),
                           (const float*)(wsb + W.dzpart), y.R, p.mfp, p.d, mtotal);
        FLURKA_CHECK_LAUNCH();
        stage_end(s, STAGE_K_BWD_MERGE);
    }
    // key side: dQ is written and dS, dz are in place
    uint16_t* img = (uint16_t*)(wsb + W.img);
    uint16_t* imgT = (uint16_t*)(wsb + W.imgT);
    {
        StageScope sc(s, STAGE_K_BWD_KEY);
        const float* Kp = a.ctx + L.Kp;
        const float* Vp = a.ctx + L.Vp;
        st = p.d == 64 ? launch_bwd_key_elu<64>(p, Kp, Vp, a.ws + GW.dS, a.ws + GW.dz, img, imgT, W.kp, s)
                       : launch_bwd_key_elu<128>(p, Kp, Vp, a.ws + GW.dS, a.ws + GW.dz, img, imgT, W.kp, s);
        if (st != FLURKA_OK) return st;
    }
    return grad_gemms(p, a, img, imgT, W.kp, (float*)(wsb + W.epart), s);
}

}  // namespace flurka
