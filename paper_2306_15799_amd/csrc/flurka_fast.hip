// bf16 MFMA path of FLuRKA attention for gfx950 (forward).
//
//   stage "project"      K' = E K, V' = F V     split-n GEMM on v_mfma_f32_32x32x16_bf16,
//                                               fp32 partial sums, deterministic second-stage sum
//   stage "key_state"    PhiK, S, z             bf16 MFMA with split-precision operands
//                                               (flurka_keystate.hip): K' enters the exponent as three
//                                               bf16 terms, because exp() turns absolute error in
//                                               omega.k' - |k'|^2/2 into relative error of the weights
//   stage "query_stream" out = (P S) / (P z)    per 32 query rows of a wavefront:
//                                               U^T = omega Q^T (MFMA) -> running row max -> exp ->
//                                               bf16 P^T kept in registers as the B operand of
//                                               N^T = S^T P^T (MFMA); the denominator on the VALU;
//                                               out and the log-denominator per row are stored
// Formulas: Eq. 2 with the App. D row normaliser; feature maps of Sec. 2, "Kernel Methods".
#include "flurka_fast.h"
#include "flurka_gemm.h"

namespace flurka {

#define FLURKA_CHECK_LAUNCH()                                   \
    do {                                                        \
        if (hipGetLastError() != hipSuccess) return FLURKA_ERR_LAUNCH; \
    } while (0)

static inline dim3 grid1d(long total, int block) { return dim3((unsigned)((total + block - 1) / block)); }

// ===========================================================================
// Stage "project": C[k x (BH*d)] = E[k x n] * X[n x (BH*d)] for X in {K, V}
// ===========================================================================
constexpr int PBM = GBM, PBN = GBN, PBK = GBK;   // tile of the shared GEMM main loop (flurka_gemm.h)

struct ProjPlan {
    int tilesM, tilesN, splits, steps_per_split, total_steps;
};

static ProjPlan proj_plan(const Problem& p) {
    ProjPlan q;
    q.tilesM = (p.k + PBM - 1) / PBM;
    const int heads_per_tile = PBN / p.d;
    q.tilesN = (p.BH + heads_per_tile - 1) / heads_per_tile;
    q.total_steps = (p.n + PBK - 1) / PBK;        // a ragged last step reads the missing positions as zero
    const int tiles = q.tilesM * q.tilesN * 2;
    int splits = chip_cus() / tiles;               // one workgroup per compute unit
    if (splits < 1) splits = 1;
    if (splits > 8) splits = splits / 8 * 8;       // keep each XCD on its own n-ranges
    if (splits > q.total_steps) splits = q.total_steps;
    q.steps_per_split = (q.total_steps + splits - 1) / splits;
    q.splits = (q.total_steps + q.steps_per_split - 1) / q.steps_per_split;
    return q;
}

// ===========================================================================
// Stage "query_stream"
// ===========================================================================
struct QueryArgs {
    const uint16_t* Q;
    const uint16_t* omega;     // (H|1, m, d)
    const uint16_t* St;        // (BH, d, mf) bf16 (performer: S_j / z_j)
    const float* zp;           // (BH, mf)
    const uint16_t* cw;        // (BH, mf, 4) bf16 terms of c + ln z (performer)
    uint16_t* out;
    float* lse;                // (BH, n) log of the denominator, kept for the backward pass
    int n, H, mf, tiles_per_head;   // mf: features incl. the padding of a ragged last tile; tiles of 32*QT rows
    int m_rows;                     // rows of omega that exist
    long total_tiles;               // BH * tiles_per_head
    long omega_head_stride;    // 0 if shared
};

template <int D>
struct QueryLds {
    // omega row: d coordinates, then one more 16-slot reduction step (the three bf16 terms of the
    // feature's exponent shift, zeros), then 16 bytes of padding
    static constexpr int w_pitch = (D + 16 + 8) * 2;
    static __host__ __device__ int s_pitch(int mf) { return (mf + 8) * 2; }
    static __host__ __device__ int w_bytes(int mf) { return mf * w_pitch; }
    static __host__ __device__ int s_bytes(int mf) { return D * s_pitch(mf); }
    static __host__ __device__ int total(int mf, int elu) {
        return (elu ? 0 : w_bytes(mf)) + s_bytes(mf) + (elu ? mf * 4 : 0) + 16;       // + z (elu1), tile counter
    }
};

// Slot of feature f (0..31) inside a 32-feature tile of the S'^T image: the order in which the first
// contraction's accumulator hands P'^T on as the B operand of the second (slot 8h + e of a group of 16
// holds feature 8*(e/4) + 4*h + e%4; the map is its own inverse).
__host__ __device__ inline int slot_of_feature_tile(int f) { return (f & 16) + 8 * ((f >> 2) & 1) + 4 * ((f >> 3) & 1) + (f & 3); }

// One workgroup = NW wavefronts sharing the LDS image of omega, S^T and z of one head; each wavefront
// streams QT tiles of 32 query rows at a time.  (QT = 2 would feed two MFMAs per operand fragment read
// from LDS, but needs more than the 256 architectural VGPRs of a wavefront; the register allocator then
// shuttles values through AGPRs and the kernel is slower than QT = 1.)
// STAGED: the Q and out tiles of a wavefront cross a private 32 x D area of LDS (placed after the
// image), so that every global access of a wavefront is 1 KiB of consecutive bytes instead of 32-byte
// pieces of 32 rows; used when the area fits beside the image (QT = 1; n is a multiple of 32 here).
// Chunk c of row r sits at chunk position c ^ ((r >> 1) & 7): conflict-free for both access patterns.
template <int D, bool ELU, int NW, int QT, bool STAGED>
__global__ __launch_bounds__(NW * 64) void query_stream_kernel(QueryArgs a) {
    static_assert(!STAGED || QT == 1, "staged tiles are one 32-row tile per wavefront");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    using L = QueryLds<D>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int mf = a.mf;
    const int s_pitch = L::s_pitch(mf);
    unsigned char* lw = lds;
    unsigned char* ls = lds + (ELU ? 0 : L::w_bytes(mf));
    float* lz = (float*)(ls + L::s_bytes(mf));                 // elu1 only
    int* const next_tile = (int*)(lz + (ELU ? mf : 0));
    constexpr int KS = D / 16;      // reduction steps over d
    constexpr int TT = D / 32;      // 32-row tiles of N^T

    // The grid is as many workgroups as the chip holds at once; each takes an equal, contiguous share
    // of all (head, 32*QT-row tile) pairs and walks it head by head, refilling the LDS image when the
    // head changes.
    const long tile_begin = a.total_tiles * blockIdx.x / gridDim.x;
    const long tile_end = a.total_tiles * (blockIdx.x + 1) / gridDim.x;
    for (long seg = tile_begin; seg < tile_end;) {
    const int bh = (int)(seg / a.tiles_per_head);
    long seg_end = (long)(bh + 1) * a.tiles_per_head;
    if (seg_end > tile_end) seg_end = tile_end;
    if (seg != tile_begin) __syncthreads();          // every wavefront is done with the previous image

    // fill the LDS image (16-byte chunks, coalesced)
    if (!ELU) {
        const uint16_t* og = a.omega + (long)(bh % a.H) * a.omega_head_stride;
        constexpr int cpr = D / 8;                      // chunks per row
        for (int c = tid; c < mf * cpr; c += NW * 64) {
            const int r = c / cpr, q = c % cpr;
            // rows of the padding: any finite row does, their shift c' of -1e30 makes the weights 0
            *(uint4*)(lw + r * L::w_pitch + 16 * q) = ld16(og + (long)(r < a.m_rows ? r : a.m_rows - 1) * D + 8 * q);
        }
        const uint16_t* cwg = a.cw + (long)bh * mf * 4;
        for (int r = tid; r < mf; r += NW * 64) {
            const uint2 t3 = *(const uint2*)(cwg + 4 * r);
            *(uint4*)(lw + r * L::w_pitch + 2 * D) = make_uint4(t3.x, t3.y, 0u, 0u);
            *(uint4*)(lw + r * L::w_pitch + 2 * D + 16) = make_uint4(0u, 0u, 0u, 0u);
        }
    }
    {
        const uint16_t* sg = a.St + (long)bh * D * mf;
        const int cpr = mf / 8;
        for (int c = tid; c < D * cpr; c += NW * 64) {
            const int r = c / cpr, q = c % cpr;
            *(uint4*)(ls + r * s_pitch + 16 * q) = ld16(sg + (long)r * mf + 8 * q);
        }
        if (ELU) {
            const float* zg = a.zp + (long)bh * mf;
            for (int c = tid; c < mf; c += NW * 64) lz[c] = zg[c];
        }
    }
    // Tiles of the segment are handed out on demand: wavefront w starts with tile w and takes the next
    // free one from this counter whenever it finishes.  (The wavefronts of a SIMD do not progress at the
    // same rate -- the older one is served first -- so a fixed split leaves the SIMD half empty at the
    // end; which wavefront computes a tile does not change its result.)
    if (tid == 0) *next_tile = NW;
    __syncthreads();

    const long head_off = (long)bh * a.n * D;
    const int row_begin = (int)(seg - (long)bh * a.tiles_per_head) * (32 * QT);
    int row_end = (int)(seg_end - (long)bh * a.tiles_per_head) * (32 * QT);
    if (row_end > a.n) row_end = a.n;
    seg = seg_end;

    // this lane's query rows (B operand of the first contraction: 8 consecutive d per step); the
    // rows of the next tile are requested while the current tile is still being worked on
    int qrow[QT];
    bool valid[QT];
    uint4 qf[QT][KS];
    constexpr int CPR = D / 8, ROWB = D * 2, LPT = 32 * CPR / 64;
    unsigned char* const scr = lds + L::total(mf, ELU) + wave * (32 * ROWB);
    auto scr_at = [&](int row, int c) -> unsigned char* { return scr + row * ROWB + 16 * (c ^ ((row >> 1) & 7)); };
    uint4 raw[LPT];                       // STAGED: the next tile as requested from memory
    auto load_queries = [&](int row0, uint4 (&dst)[QT][KS]) {
        if constexpr (STAGED) {
#pragma unroll
            for (int u = 0; u < LPT; ++u) raw[u] = ld16(a.Q + head_off + (long)row0 * D + 8 * lane + 512 * u);
        } else {
#pragma unroll
            for (int i = 0; i < QT; ++i) {
                int r = row0 + 32 * i + l32;
                if (r >= a.n) r = a.n - 1;
                const uint16_t* qg = a.Q + head_off + (long)r * D + 8 * half;
#pragma unroll
                for (int s = 0; s < KS; ++s) dst[i][s] = ld16(qg + 16 * s);
            }
        }
    };
    const int row_first = row_begin + 32 * QT * wave;
    if (row_first < row_end) load_queries(row_first, qf);

    for (int row0 = row_first; row0 < row_end;) {
        floatx16 accN[QT][TT];
        float den[QT];
        int grabbed = 0;
        if (lane == 0) grabbed = atomicAdd(next_tile, 1);
        const int row_next = row_begin + 32 * QT * __builtin_amdgcn_readfirstlane(grabbed);
#pragma unroll
        for (int i = 0; i < QT; ++i) {
            qrow[i] = row0 + 32 * i + l32;
            if constexpr (STAGED) {
#pragma unroll
                for (int u = 0; u < LPT; ++u) *(uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR) = raw[u];
#pragma unroll
                for (int s = 0; s < KS; ++s) qf[i][s] = *(const uint4*)scr_at(l32, 2 * s + half);
            }
            valid[i] = qrow[i] < a.n;
            if (!valid[i]) qrow[i] = a.n - 1;
#pragma unroll
            for (int t = 0; t < TT; ++t) accN[i][t] = zero16();
            den[i] = 0.f;
        }

        float mu[QT];     // running row maxima (same value in lanes l and l^32); 0 for elu1
#pragma unroll
        for (int i = 0; i < QT; ++i) mu[i] = ELU ? 0.f : -INFINITY;
        if (ELU) {
            // P = elu(q)+1 straight in operand order; features are the d coordinates
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                uint4 pb[QT];
#pragma unroll
                for (int i = 0; i < QT; ++i) {
                    const uint32_t w[4] = {qf[i][s].x, qf[i][s].y, qf[i][s].z, qf[i][s].w};
                    uint32_t pk[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x0 = bf16_to_f32((uint16_t)(w[e] & 0xffffu));
                        const float x1 = bf16_to_f32((uint16_t)(w[e] >> 16));
                        const float p0 = x0 > 0.f ? x0 + 1.f : __expf(x0);
                        const float p1 = x1 > 0.f ? x1 + 1.f : __expf(x1);
                        pk[e] = pack_bf16(p0, p1);
                        const int f = 16 * s + 8 * half + 2 * e;
                        den[i] = fmaf(p0, lz[f], den[i]);
                        den[i] = fmaf(p1, lz[f + 1], den[i]);
                    }
                    pb[i] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                }
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    const uint4 sa = *(const uint4*)(ls + (32 * t + l32) * s_pitch + 32 * s + 16 * half);
#pragma unroll
                    for (int i = 0; i < QT; ++i) accN[i][t] = mfma32(sa, pb[i], accN[i][t]);
                }
                __builtin_amdgcn_sched_barrier(0);        // keeps the unrolled steps from piling up loads
            }
            if (row_next < row_end) load_queries(row_next, qf);
        } else {
            forward_feature_pass<D, QT>(lw, L::w_pitch, ls, s_pitch, mf / 32, l32, half, qf, accN, den, mu,
                                        [&] { if (row_next < row_end) load_queries(row_next, qf); });
        }
#pragma unroll
        for (int i = 0; i < QT; ++i) {
            const float dsum = half_sum(den[i]);
            const float inv = 1.f / dsum;
            if (valid[i]) {
                if (half == 0) a.lse[(long)bh * a.n + qrow[i]] = mu[i] + __logf(dsum);
                uint16_t* og = a.out + head_off + (long)qrow[i] * D;
#pragma unroll
                for (int t = 0; t < TT; ++t)
#pragma unroll
                    for (int q = 0; q < 4; q += 2) {
                        uint2 ev, od;
                        ev.x = pack_bf16(accN[i][t][4 * q] * inv, accN[i][t][4 * q + 1] * inv);
                        ev.y = pack_bf16(accN[i][t][4 * q + 2] * inv, accN[i][t][4 * q + 3] * inv);
                        od.x = pack_bf16(accN[i][t][4 * q + 4] * inv, accN[i][t][4 * q + 5] * inv);
                        od.y = pack_bf16(accN[i][t][4 * q + 6] * inv, accN[i][t][4 * q + 7] * inv);
                        if constexpr (STAGED) *(uint4*)scr_at(l32, 4 * t + q + half) = join_halves(ev, od);
                        else                  *(uint4*)(og + 32 * t + 8 * (q + half)) = join_halves(ev, od);
                    }
            }
            if constexpr (STAGED) {
                uint16_t* ob = a.out + head_off + (long)row0 * D + 8 * lane;
#pragma unroll
                for (int u = 0; u < LPT; ++u)
                    *(uint4*)(ob + 512 * u) = *(const uint4*)scr_at((64 * u + lane) / CPR, (64 * u + lane) % CPR);
            }
        }
        row0 = row_next;
    }
    }   // head segments
}

// ===========================================================================
// Host side
// ===========================================================================
static int query_lds_bytes(const Problem& p) {
    return p.d == 64 ? QueryLds<64>::total(p.mfp, p.elu) : QueryLds<128>::total(p.mfp, p.elu);
}

bool fast_supported(const Problem& p, int bwd) {
    if (bwd) return fast_bwd_supported(p);
    if (!p.bf16) return false;
    if (p.d != 64 && p.d != 128) return false;
    if (p.n % 8 != 0) return false;                // rows of E and F start on 16-byte boundaries
    if (query_lds_bytes(p) > 160 * 1024) return false;
    // 32-bit byte offsets inside the projection's buffer descriptors
    if (((size_t)p.k + PBM) * (size_t)p.n * 2 >= ((size_t)1 << 31)) return false;
    if ((size_t)(PBN / p.d) * (size_t)p.n * (size_t)p.d * 2 >= ((size_t)1 << 31)) return false;
    return true;
}

bool fast_pointers_ok(const void* a, const void* b, const void* c, const void* d, const void* e,
                      const void* f, const void* g) {
    const void* ps[7] = {a, b, c, d, e, f, g};
    for (const void* p : ps)
        if (p && ((uintptr_t)p % 16) != 0) return false;
    return true;
}

struct FastWs {
    size_t partial, Kimg, Vimg, nrm, St, zp, cw, total;    // byte offsets
};

static FastWs fast_ws_layout(const Problem& p) {
    FastWs W{};
    const ProjPlan q = proj_plan(p);
    const KeyStatePlan ks = key_state_plan(p);
    const size_t BH = (size_t)p.BH;
    size_t o = 0;
    // tile-ordered fp32 partials of K' and V', one set per split
    W.partial = o; o += round_up((size_t)2 * q.splits * q.tilesM * q.tilesN * G_TILE_ELEMS * 4, 256);
    W.Kimg = o;    o += round_up(p.elu ? 0 : 3 * BH * ks.kpad * p.d * 2, 256);
    W.Vimg = o;    o += round_up(2 * BH * (ks.kpad / 2) * p.d * 4, 256);
    W.nrm = o;     o += round_up(BH * ks.kpad * 4, 256);
    W.St = o;      o += round_up(BH * p.d * p.mfp * 2, 256);
    W.zp = o;      o += round_up(BH * p.mfp * 4, 256);
    W.cw = o;      o += round_up(BH * p.mfp * 8, 256);
    W.total = o;
    return W;
}

size_t fast_ws_bytes(const Problem& p, int bwd) {
    return bwd ? fast_bwd_ws_bytes(p) : fast_ws_layout(p).total;
}

constexpr int QS_QT = 1;                  // 32-row tiles per wavefront
// wavefronts per workgroup: as many per SIMD as the register budget of the kernel allows
template <int D> struct QsWaves { static constexpr int value = D == 64 ? 12 : 8; };

template <int D, bool ELU, bool STAGED>
static flurka_status launch_query_impl(const QueryArgs& qa, int ldsb, hipStream_t s) {
    constexpr int QS_NW = QsWaves<D>::value;
    auto kern = query_stream_kernel<D, ELU, QS_NW, QS_QT, STAGED>;
    const int grid = resident_grid((const void*)kern, QS_NW * 64, ldsb, qa.total_tiles);
    if (grid < 1) return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(QS_NW * 64), ldsb, s, qa);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

// The LDS image alone must fit (fast_supported).  The staged tiles are used for the elu1 map when they
// fit beside it: that kernel is bound by its Q and out traffic (measured: 71 -> 49 us at n = 16384,
// B*H = 64); with the random-feature map the kernel is not, and the extra registers cost as much as the
// better access pattern gains.
template <int D, bool ELU>
static flurka_status launch_query(const Problem& p, const QueryArgs& qa, int ldsb, hipStream_t s) {
    if constexpr (ELU && QS_QT == 1) {
        const int staged = ldsb + QsWaves<D>::value * 32 * D * 2;
        if (p.n % 32 == 0 && staged <= 160 * 1024) return launch_query_impl<D, ELU, true>(qa, staged, s);
    }
    return launch_query_impl<D, ELU, false>(qa, ldsb, s);
}

// Query stream over the St / zp / cw images the key-state stage left in the workspace.
static flurka_status run_query_stream(const Problem& p, const void* Q, const void* omega, void* out, float* lse,
                                      const uint16_t* St, const float* zp, const uint16_t* cw, hipStream_t s) {
    StageScope sc(s, STAGE_K_QUERY_STREAM);
    QueryArgs qa{};
    qa.Q = (const uint16_t*)Q;
    qa.omega = (const uint16_t*)omega;
    qa.St = St;
    qa.zp = zp;
    qa.cw = cw;
    qa.out = (uint16_t*)out;
    qa.lse = lse;
    qa.n = p.n; qa.H = p.H; qa.mf = p.mfp; qa.m_rows = p.mf;
    qa.omega_head_stride = p.omega_per_head ? (long)p.m * p.d : 0;
    qa.tiles_per_head = (p.n + 32 * QS_QT - 1) / (32 * QS_QT);
    qa.total_tiles = (long)p.BH * qa.tiles_per_head;
    const int ldsb = query_lds_bytes(p);
    if (p.d == 64)
        return p.elu ? launch_query<64, true>(p, qa, ldsb, s) : launch_query<64, false>(p, qa, ldsb, s);
    return p.elu ? launch_query<128, true>(p, qa, ldsb, s) : launch_query<128, false>(p, qa, ldsb, s);
}

flurka_status fast_forward(const Problem& p, const FwdArgs& a, hipStream_t s) {
    const FastWs W = fast_ws_layout(p);
    unsigned char* wsb = (unsigned char*)a.ws;
    flurka_status st;
    int proj_splits = 1;
    {
        StageScope sc(s, STAGE_K_PROJ_GEMM);
        const ProjPlan q = proj_plan(p);
        GemmParams gp{};
        gp.A[0] = (const uint16_t*)a.E; gp.A[1] = (const uint16_t*)a.F;
        gp.B[0] = (const uint16_t*)a.K; gp.B[1] = (const uint16_t*)a.V;
        gp.C[0] = wsb + W.partial;
        gp.C[1] = nullptr;
        gp.n = p.n; gp.d = p.d; gp.k = p.k; gp.BH = p.BH; gp.kp = p.k;
        gp.tilesM = q.tilesM; gp.tilesN = q.tilesN; gp.splits = q.splits;
        gp.steps_per_split = q.steps_per_split; gp.total_steps = q.total_steps;
        st = p.d == 64 ? launch_gemm_mfma<ProjPolicy<64>>(gp, s) : launch_gemm_mfma<ProjPolicy<128>>(gp, s);
        if (st != FLURKA_OK) return st;
        proj_splits = q.splits;
    }
    {
        KeyStateBuffers kb{};
        kb.Kimg = (uint16_t*)(wsb + W.Kimg); kb.Vimg = (uint32_t*)(wsb + W.Vimg); kb.nrm = (float*)(wsb + W.nrm);
        kb.St = (uint16_t*)(wsb + W.St); kb.zp = (float*)(wsb + W.zp); kb.cw = (uint16_t*)(wsb + W.cw);
        const ProjPlan q = proj_plan(p);
        st = fast_key_state(p, a.omega, a.ctx, (const float*)(wsb + W.partial), q.tilesM, q.tilesN, proj_splits, kb, s);
        if (st != FLURKA_OK) return st;
    }
    return run_query_stream(p, a.Q, a.omega, a.out, a.ctx + ctx_layout(p).lse, (const uint16_t*)(wsb + W.St),
                            (const float*)(wsb + W.zp), (const uint16_t*)(wsb + W.cw), s);
}

// ===========================================================================
// Paper-order path: K' = (E X_K) W^K, V' = (F X_V) W^V  (Eq. 2 read literally: the sequence projection
// is applied to the model-wide layer input, the per-head transform to its k projected rows)
// ===========================================================================
// Y = E X from the first product's split partials -> the three-term bf16 image of Y that the second
// product reads as its A operand: image[which][batch][row][term][column], term = hi, mid, lo.
// One wavefront per (which, batch, four rows, 64 columns); a lane's four rows are the four floats of
// one 16-byte element of the tile-ordered partials.
struct WideFinishArgs {
    const float* part;
    uint16_t* img;
    int splits, tilesM, tilesN, tiles_per_batch, k, dm, B;
};

__global__ __launch_bounds__(256) void wide_finish_kernel(WideFinishArgs a) {
    const int lane = threadIdx.x & 63;
    long wid = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int col_chunks = (a.dm + 63) / 64, row_groups = (a.k + 3) / 4;
    if (wid >= (long)2 * a.B * row_groups * col_chunks) return;
    const int cc = (int)(wid % col_chunks); wid /= col_chunks;
    const int rg = (int)(wid % row_groups); wid /= row_groups;
    const int b = (int)(wid % a.B);
    const int which = (int)(wid / a.B);
    const int c = 64 * cc + lane, r0 = 4 * rg;
    if (c >= a.dm) return;
    const int tn = b * a.tiles_per_batch + c / GBN, tm = r0 / GBM;
    const int eo = partial_elem_offset(r0 % GBM, c % GBN);
    float4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < a.splits; ++s) {
        const float4 x = *(const float4*)(a.part + partial_tile_index(which, s, tn, tm, a.splits, a.tilesN, a.tilesM) * G_TILE_ELEMS + eo);
        sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
    }
    const float v[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (r0 + e >= a.k) break;
        uint32_t hi, mid, lo;
        split3_pair(v[e], 0.f, hi, mid, lo);
        uint16_t* row = a.img + (((long)(which * a.B + b) * a.k + r0 + e) * 3) * a.dm + c;
        row[0] = (uint16_t)hi;
        row[a.dm] = (uint16_t)mid;
        row[2 * a.dm] = (uint16_t)lo;
    }
}

struct SplitPlan { int splits, steps_per_split; };
// split of a reduction of `total_steps` steps so that `tiles` output tiles give about one workgroup per
// compute unit (the rule of proj_plan)
static SplitPlan split_plan(int tiles, int total_steps) {
    int splits = chip_cus() / tiles;
    if (splits < 1) splits = 1;
    if (splits > 8) splits = splits / 8 * 8;
    if (splits > total_steps) splits = total_steps;
    SplitPlan q;
    q.steps_per_split = (total_steps + splits - 1) / splits;
    q.splits = (total_steps + q.steps_per_split - 1) / q.steps_per_split;
    return q;
}

struct FusedWPlan {
    int tilesM, tpb1, tilesN1, steps1, tpb2, tilesN2, steps2;
    SplitPlan s1, s2;
};

static FusedWPlan fusedw_plan(const Problem& p, int dm) {
    FusedWPlan q;
    q.tilesM = (p.k + GBM - 1) / GBM;
    q.tpb1 = (dm + GBN - 1) / GBN;
    q.tilesN1 = p.B * q.tpb1;
    q.steps1 = (p.n + GBK - 1) / GBK;
    q.s1 = split_plan(q.tilesM * q.tilesN1 * 2, q.steps1);
    q.tpb2 = p.H * p.d / GBN;
    q.tilesN2 = p.B * q.tpb2;
    q.steps2 = 3 * dm / GBK;
    q.s2 = split_plan(q.tilesM * q.tilesN2 * 2, q.steps2);
    return q;
}

bool fast_fusedw_supported(const Problem& p, int dm) {
    if (!fast_supported(p, 0)) return false;
    if (dm < GBK || dm % GBK != 0) return false;             // whole reduction steps of the second product
    if ((p.H * p.d) % GBN != 0) return false;                // column tiles of the second product inside one batch
    // 32-bit byte offsets inside the buffer descriptors of the two products
    if ((size_t)p.n * dm * 2 >= ((size_t)1 << 31)) return false;
    if (((size_t)p.k + GBM) * 3 * dm * 2 >= ((size_t)1 << 31)) return false;
    if (((size_t)p.H * p.d + GBN) * dm * 2 >= ((size_t)1 << 31)) return false;
    return true;
}

struct FusedWWs { size_t partial, img, rest, total; };

static FusedWWs fusedw_ws_layout(const Problem& p, int dm) {
    const FusedWPlan q = fusedw_plan(p, dm);
    FusedWWs W{};
    const size_t p1 = (size_t)2 * q.s1.splits * q.tilesM * q.tilesN1 * G_TILE_ELEMS * 4;
    const size_t p2 = (size_t)2 * q.s2.splits * q.tilesM * q.tilesN2 * G_TILE_ELEMS * 4;
    size_t o = 0;
    W.partial = o; o += round_up(p1 > p2 ? p1 : p2, 256);    // the second product reuses the first one's room
    W.img = o;     o += round_up((size_t)2 * p.B * p.k * 3 * dm * 2, 256);
    W.rest = o;    o += fast_ws_layout(p).total;             // key-state and query-stream images (its `partial` part unused)
    W.total = o;
    return W;
}

size_t fast_fusedw_ws_bytes(const Problem& p, int dm) { return fusedw_ws_layout(p, dm).total; }

flurka_status fast_forward_fusedw(const Problem& p, const FusedWArgs& a, hipStream_t s) {
    const FusedWPlan q = fusedw_plan(p, a.dm);
    const FusedWWs W = fusedw_ws_layout(p, a.dm);
    const FastWs R = fast_ws_layout(p);
    unsigned char* wsb = (unsigned char*)a.ws;
    unsigned char* rest = wsb + W.rest;
    flurka_status st;
    {
        StageScope sc(s, STAGE_K_WIDE_GEMM);
        GemmParams gp{};
        gp.A[0] = (const uint16_t*)a.E; gp.A[1] = (const uint16_t*)a.F;
        gp.B[0] = (const uint16_t*)a.XK; gp.B[1] = (const uint16_t*)a.XV;
        gp.C[0] = wsb + W.partial;
        gp.n = p.n; gp.d = p.d; gp.k = p.k; gp.BH = p.BH; gp.kp = p.k;
        gp.dm = a.dm; gp.tiles_per_batch = q.tpb1;
        gp.tilesM = q.tilesM; gp.tilesN = q.tilesN1; gp.splits = q.s1.splits;
        gp.steps_per_split = q.s1.steps_per_split; gp.total_steps = q.steps1;
        if ((st = launch_gemm_mfma<ProjWidePolicy>(gp, s)) != FLURKA_OK) return st;
    }
    {
        StageScope sc(s, STAGE_K_WIDE_FINISH);
        WideFinishArgs fa{};
        fa.part = (const float*)(wsb + W.partial); fa.img = (uint16_t*)(wsb + W.img);
        fa.splits = q.s1.splits; fa.tilesM = q.tilesM; fa.tilesN = q.tilesN1; fa.tiles_per_batch = q.tpb1;
        fa.k = p.k; fa.dm = a.dm; fa.B = p.B;
        const long waves = (long)2 * p.B * ((p.k + 3) / 4) * ((a.dm + 63) / 64);
        hipLaunchKernelGGL(wide_finish_kernel, grid1d(waves, 4), dim3(256), 0, s, fa);
        FLURKA_CHECK_LAUNCH();
    }
    {
        StageScope sc(s, STAGE_K_TRANSFORM_GEMM);
        const size_t img_elems = (size_t)p.B * p.k * 3 * a.dm;
        GemmParams gp{};
        gp.A[0] = (const uint16_t*)(wsb + W.img); gp.A[1] = gp.A[0] + img_elems;
        gp.B[0] = (const uint16_t*)a.WK; gp.B[1] = (const uint16_t*)a.WV;
        gp.C[0] = wsb + W.partial;
        gp.n = p.n; gp.d = p.d; gp.k = p.k; gp.BH = p.BH; gp.kp = p.k;
        gp.dm = a.dm; gp.tiles_per_batch = q.tpb2;
        gp.tilesM = q.tilesM; gp.tilesN = q.tilesN2; gp.splits = q.s2.splits;
        gp.steps_per_split = q.s2.steps_per_split; gp.total_steps = q.steps2;
        if ((st = launch_gemm_mfma<TransformPolicy>(gp, s)) != FLURKA_OK) return st;
    }
    KeyStateBuffers kb{};
    kb.Kimg = (uint16_t*)(rest + R.Kimg); kb.Vimg = (uint32_t*)(rest + R.Vimg); kb.nrm = (float*)(rest + R.nrm);
    kb.St = (uint16_t*)(rest + R.St); kb.zp = (float*)(rest + R.zp); kb.cw = (uint16_t*)(rest + R.cw);
    st = fast_key_state(p, a.omega, a.ctx, (const float*)(wsb + W.partial), q.tilesM, q.tilesN2, q.s2.splits, kb, s);
    if (st != FLURKA_OK) return st;
    return run_query_stream(p, a.Q, a.omega, a.out, a.ctx + ctx_layout(p).lse, kb.St, kb.zp, kb.cw, s);
}

// ===========================================================================
// Comparison baselines at the attention level (the paper's constituents, Sec. 2): kernel attention
// without a sequence projection, and Linformer's softmax over the k projected keys.  Both reuse the
// kernels above; they exist so that the speed comparisons of Sec. 4.1 / 4.3 can be run on this hardware.
// ===========================================================================
// Kernel attention phi(Q)(phi(K)^T V) / phi(Q)(phi(K)^T 1): FLuRKA with E = F = I, computed without the
// n x n product.  `p` has k == n.  ctx: S, z, c, lse at the offsets of the same problem with k = 1.
static Problem ctx_problem_kernel_attn(const Problem& p) { Problem q = p; q.k = 1; return q; }

struct KernelAttnWs { size_t Kimg, Vimg, nrm, St, zp, cw, total; };
static KernelAttnWs kernel_attn_ws_layout(const Problem& p) {
    KernelAttnWs W{};
    const size_t BH = (size_t)p.BH;
    size_t o = 0;
    W.Kimg = o; o += round_up(p.elu ? 0 : BH * p.n * p.d * 2, 256);
    W.Vimg = o; o += round_up(BH * (p.n / 2) * p.d * 4, 256);
    W.nrm = o;  o += round_up(BH * p.n * 4, 256);
    W.St = o;   o += round_up(BH * p.d * p.mfp * 2, 256);
    W.zp = o;   o += round_up(BH * p.mfp * 4, 256);
    W.cw = o;   o += round_up(BH * p.mfp * 8, 256);
    W.total = o;
    return W;
}

// Linformer: softmax(Q K'^T) V' over the k projected keys.  With omega := K' (one "feature" per key, rounded
// to bf16), S' := V' and zero shifts the query stream computes exactly that: u = K' q, running row maximum,
// exp, P V' / sum P.  linformer_pack writes those images from K', V' in ctx; keys past k (k is padded to
// whole 32-key tiles) get the shift -inf, i.e. weight 0.
__global__ void linformer_pack_kernel(const float* Kp, const float* Vp, uint16_t* Wimg, uint16_t* St, uint16_t* cw,
                                      int k, int kpad, int d, long total) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;        // (bh, r < kpad, t)
    if (idx >= total) return;
    const int t = (int)(idx % d);
    const long rest = idx / d;
    const int r = (int)(rest % kpad);
    const long bh = rest / kpad;
    const bool live = r < k;
    const float kv = live ? Kp[(bh * k + r) * d + t] : 0.f;
    const float vv = live ? Vp[(bh * k + r) * d + t] : 0.f;
    Wimg[(bh * kpad + r) * d + t] = f32_to_bf16(kv);
    St[(bh * d + t) * kpad + (r & ~31) + slot_of_feature_tile(r & 31)] = f32_to_bf16(vv);
    if (t < 4) cw[(bh * kpad + r) * 4 + t] = (t == 0 && !live) ? (uint16_t)0xff80u : (uint16_t)0;
}

static Problem query_problem_linformer(const Problem& p) {
    Problem q = p;
    q.m = q.mf = q.mfp = (p.k + 31) / 32 * 32;     // one feature per projected key
    q.H = p.BH; q.B = 1;                   // every (batch, head) has its own K'
    q.omega_per_head = 1;
    q.elu = 0;
    return q;
}

struct LinformerWs { size_t partial, Wimg, St, zp, cw, total; };
static LinformerWs linformer_ws_layout(const Problem& p) {
    LinformerWs W{};
    const ProjPlan q = proj_plan(p);
    const size_t BH = (size_t)p.BH, kpad = (size_t)(p.k + 31) / 32 * 32;
    size_t o = 0;
    W.partial = o; o += round_up((size_t)2 * q.splits * q.tilesM * q.tilesN * G_TILE_ELEMS * 4, 256);
    W.Wimg = o;    o += round_up(BH * kpad * p.d * 2, 256);
    W.St = o;      o += round_up(BH * p.d * kpad * 2, 256);
    W.zp = o;      o += round_up(BH * kpad * 4, 256);
    W.cw = o;      o += round_up(BH * kpad * 8, 256);
    W.total = o;
    return W;
}

bool fast_baseline_supported(int which, const Problem& p) {
    if (!p.bf16 || (p.d != 64 && p.d != 128) || p.n % PBK != 0) return false;
    if (which == FLURKA_BASELINE_KERNEL_ATTN) {
        if (p.k != p.n || p.mf % 32 != 0) return false;
        if (query_lds_bytes(p) > 160 * 1024) return false;
        return (size_t)p.BH * p.n * p.d * 2 < ((size_t)1 << 40);
    }
    if (which == FLURKA_BASELINE_LINFORMER) {
        if (p.elu) return false;
        if (!fast_supported(p, 0)) return false;                       // the projection's limits
        return query_lds_bytes(query_problem_linformer(p)) <= 160 * 1024;   // K', V' of a head in LDS
    }
    return false;
}

size_t fast_baseline_ws_bytes(int which, const Problem& p) {
    return which == FLURKA_BASELINE_KERNEL_ATTN ? kernel_attn_ws_layout(p).total : linformer_ws_layout(p).total;
}

size_t fast_baseline_ctx_floats(int which, const Problem& p) {
    return which == FLURKA_BASELINE_KERNEL_ATTN ? ctx_layout(ctx_problem_kernel_attn(p)).total : ctx_layout(p).total;
}

flurka_status fast_kernel_attn_forward(const Problem& p, const FwdArgs& a, hipStream_t s) {
    const KernelAttnWs W = kernel_attn_ws_layout(p);
    const CtxLayout L = ctx_layout(ctx_problem_kernel_attn(p));
    unsigned char* wsb = (unsigned char*)a.ws;
    KeyStateBuffers kb{};
    kb.Kimg = (uint16_t*)(wsb + W.Kimg); kb.Vimg = (uint32_t*)(wsb + W.Vimg); kb.nrm = (float*)(wsb + W.nrm);
    kb.St = (uint16_t*)(wsb + W.St); kb.zp = (float*)(wsb + W.zp); kb.cw = (uint16_t*)(wsb + W.cw);
    const flurka_status st = fast_identity_key_state(p, a.K, a.V, a.omega, a.ctx + L.S, a.ctx + L.z, a.ctx + L.c, kb, s);
    if (st != FLURKA_OK) return st;
    return run_query_stream(p, a.Q, a.omega, a.out, a.ctx + L.lse, kb.St, kb.zp, kb.cw, s);
}

flurka_status fast_linformer_forward(const Problem& p, const FwdArgs& a, hipStream_t s) {
    const LinformerWs W = linformer_ws_layout(p);
    const CtxLayout L = ctx_layout(p);
    const ProjPlan q = proj_plan(p);
    unsigned char* wsb = (unsigned char*)a.ws;
    flurka_status st;
    {
        StageScope sc(s, STAGE_K_PROJ_GEMM);
        GemmParams gp{};
        gp.A[0] = (const uint16_t*)a.E; gp.A[1] = (const uint16_t*)a.F;
        gp.B[0] = (const uint16_t*)a.K; gp.B[1] = (const uint16_t*)a.V;
        gp.C[0] = wsb + W.partial;
        gp.n = p.n; gp.d = p.d; gp.k = p.k; gp.BH = p.BH; gp.kp = p.k;
        gp.tilesM = q.tilesM; gp.tilesN = q.tilesN; gp.splits = q.splits;
        gp.steps_per_split = q.steps_per_split; gp.total_steps = q.total_steps;
        st = p.d == 64 ? launch_gemm_mfma<ProjPolicy<64>>(gp, s) : launch_gemm_mfma<ProjPolicy<128>>(gp, s);
        if (st != FLURKA_OK) return st;
    }
    KeyStateBuffers none{};
    if ((st = fast_proj_finish(p, a.ctx, (const float*)(wsb + W.partial), q.tilesM, q.tilesN, q.splits, false, none, s)) != FLURKA_OK)
        return st;
    const Problem pq = query_problem_linformer(p);
    {
        StageScope sc(s, STAGE_K_LINFORMER_PACK);
        const long total = (long)p.BH * pq.mf * p.d;
        hipLaunchKernelGGL(linformer_pack_kernel, grid1d(total, 256), dim3(256), 0, s, (const float*)(a.ctx + L.Kp),
                           (const float*)(a.ctx + L.Vp), (uint16_t*)(wsb + W.Wimg), (uint16_t*)(wsb + W.St),
                           (uint16_t*)(wsb + W.cw), p.k, pq.mf, p.d, total);
        FLURKA_CHECK_LAUNCH();
    }
    return run_query_stream(pq, a.Q, wsb + W.Wimg, a.out, a.ctx + L.lse, (const uint16_t*)(wsb + W.St),
                            (const float*)(wsb + W.zp), (const uint16_t*)(wsb + W.cw), s);
}

}  // namespace flurka
