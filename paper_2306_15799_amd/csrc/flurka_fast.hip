// bf16 MFMA path of FLuRKA attention for gfx950 (forward).
//
//   stage "project"      K' = E K, V' = F V     split-n GEMM on v_mfma_f32_32x32x16_bf16,
//                                               fp32 partial sums, deterministic second-stage sum
//   stage "key_state"    PhiK, S, z             fp32 kernels shared with the generic path (K' must stay
//                                               fp32 into the exponent: exp() turns absolute error in
//                                               omega.k' - |k'|^2/2 into relative error of the weights)
//   stage "query_stream" out = (P S) / (P z)    per 32 query rows of a wavefront:
//                                               U^T = omega Q^T (MFMA) -> running row max -> exp ->
//                                               bf16 P^T kept in registers as the B operand of
//                                               N^T = S^T P^T (MFMA); the denominator on the VALU
// Formulas: Eq. 2 with the App. D row normaliser; feature maps of Sec. 2, "Kernel Methods".
#include "flurka_fast.h"

namespace flurka {

#define FLURKA_CHECK_LAUNCH()                                   \
    do {                                                        \
        if (hipGetLastError() != hipSuccess) return FLURKA_ERR_LAUNCH; \
    } while (0)

static inline dim3 grid1d(long total, int block) { return dim3((unsigned)((total + block - 1) / block)); }

// ===========================================================================
// Stage "project": C[k x (BH*d)] = E[k x n] * X[n x (BH*d)] for X in {K, V}
// ===========================================================================
constexpr int PBM = 256;              // rows of E per workgroup
constexpr int PBN = 256;              // columns (whole heads) per workgroup
constexpr int PBK = 64;               // sequence positions per main-loop step
constexpr int PA_PITCH = 144;         // bytes per LDS row of the E tile (128 + 16 pad: conflict-free b128 reads)
constexpr int PA_STAGE = PBM * PA_PITCH;
// X tile in LDS: [group of 8 positions][column][8 positions] bf16, i.e. every column's 8 consecutive
// positions form one 16-byte MFMA operand chunk.  Within a plane the chunk of column c sits at
// position c ^ ((c >> 4) & 15): a thread writes columns 8*cg + j for j = 0..7 one instruction at a
// time, so without the swizzle the lanes of one write would be 128 bytes apart and hit two banks
constexpr int PB_STAGE = (PBK / 8) * PBN * 16;
constexpr int P_STAGE = PA_STAGE + PB_STAGE;
constexpr int P_LDS = 2 * P_STAGE;    // double buffered: 139,264 bytes

struct ProjArgs {
    const uint16_t* EF[2];    // E, F
    const uint16_t* X[2];     // K, V
    float* out[2];            // destination of split 0 for K', V'; split s adds s * split_stride
    long split_stride;        // floats
    int n, d, k, BH;
    int tilesM, tilesN, splits, steps_per_split, total_steps;
};

template <int N>
struct IC { static constexpr int value = N; };

// Main loop structure (one wavefront per SIMD, so every latency has to be hidden inside the
// instruction stream of that one wavefront): a 64-position step is four 16-position sub-steps of
// 16 MFMAs each.  While sub-step s multiplies, the operand fragments of sub-step s+1 are read from
// LDS into the other register set; the global loads of the next step are issued during sub-step 0,
// transposed and written to the other LDS buffer during sub-step 2, the single barrier of the step
// sits between sub-steps 2 and 3, and sub-step 3 already prefetches from the next buffer.
// sched_barrier(0) after every "2 MFMA + 1..4 other" group keeps the compiler from undoing this.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16-byte load through a buffer descriptor: per-thread byte offset + wave-uniform byte offset;
// addresses past the descriptor's range read as zero
__device__ __forceinline__ uint4 buf_ld16(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <int D>
__global__ __launch_bounds__(256) void proj_mfma_kernel(ProjArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int half = lane >> 5, l32 = lane & 31;

    // workgroup -> (split, row tile, column tile, which); consecutive ids walk the splits first, so
    // with a split count that is a multiple of 8 every XCD (ids mod 8) keeps to its own n-ranges
    int id = blockIdx.x;
    const int split = id % a.splits; id /= a.splits;
    const int tm = id % a.tilesM;    id /= a.tilesM;
    const int tn = id % a.tilesN;    id /= a.tilesN;
    const int which = id;
    const uint16_t* __restrict__ Eg = a.EF[which];
    const uint16_t* __restrict__ Xg = a.X[which];
    const int m0 = tm * PBM;
    constexpr int heads_per_tile = PBN / D;
    const int bh0 = tn * heads_per_tile;
    const int step0 = split * a.steps_per_split;
    int step1 = step0 + a.steps_per_split;
    if (step1 > a.total_steps) step1 = a.total_steps;

    // Global reads go through buffer descriptors: rows of E past k and heads past BH fall outside the
    // descriptor and read as zero (such rows/columns are computed but never stored).
    const __amdgpu_buffer_rsrc_t rsA =
        __builtin_amdgcn_make_buffer_rsrc((void*)Eg, 0, (int)((unsigned)a.k * (unsigned)a.n * 2u), 0x00020000);
    int tile_heads = a.BH - bh0;
    if (tile_heads > heads_per_tile) tile_heads = heads_per_tile;
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(Xg + (long)bh0 * a.n * D), 0, (int)((unsigned)tile_heads * (unsigned)a.n * (unsigned)(D * 2)),
        0x00020000);
    const int a_chunk = tid & 7;                 // 16-byte chunk within a 128-byte row segment
    const int voffA = ((m0 + (tid >> 3)) * a.n + 8 * a_chunk) * 2;      // + q * 32 rows (uniform), + step
    const int rowsA = 64 * a.n;                                          // bytes between rows r and r + 32
    const int b_cg = tid & 31;                   // group of 8 columns
    const int b_kg = tid >> 5;                   // group of 8 positions
    const int b_col = 8 * b_cg;
    const int voffB = (((b_col / D) * a.n + 8 * b_kg) * D + (b_col % D)) * 2;   // + q rows (immediate), + step

    // LDS addresses of this thread's writes and of this lane's operand reads (per buffer: + P_STAGE)
    unsigned char* const a_dst = lds + (tid >> 3) * PA_PITCH + 16 * a_chunk;                 // + 32*u rows
    const int b_dst0 = PA_STAGE + (b_kg * PBN + (b_col & ~15) + ((8 * (b_cg & 1)) ^ ((b_cg >> 1) & 15))) * 16;  // ^ 16*c
    const unsigned char* const fa_src = lds + (wm * 128 + l32) * PA_PITCH + 16 * half;       // + 32*i rows, + 32*s
    const unsigned char* fb_src[4];                                                          // + 2*s planes
    {
        const int c0 = wn * 128 + (l32 & 16) + ((l32 & 15) ^ ((8 * wn + (l32 >> 4)) & 15));
#pragma unroll
        for (int j = 0; j < 4; ++j) fb_src[j] = lds + PA_STAGE + (half * PBN + ((c0 ^ (2 * j)) + 32 * j)) * 16;
    }

    // Staging registers: two whole steps of global data are in flight per workgroup (2 x 64 KB),
    // which is what it takes to cover HBM latency with one workgroup per compute unit.
    uint4 RA[2][8], RB[2][8];
    uint4 FA[2][4], FB[2][4];
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = zero16();

#define PROJ_SB() __builtin_amdgcn_sched_barrier(0)
#define PROJ_MMA(set, i, j) acc[i][j] = mfma32(FA[set][i], FB[set][j], acc[i][j])
#define PROJ_LDA(set, buf, s, i) \
    FA[set][i] = *(const uint4*)(fa_src + (buf) * P_STAGE + (32 * (i)) * PA_PITCH + 32 * (s))
#define PROJ_LDB(set, buf, s, j) \
    FB[set][j] = *(const uint4*)(fb_src[j] + (buf) * P_STAGE + ((2 * (s)) * PBN) * 16)

    // transposes 8 positions x 8 columns held in rb[0..7] and stores column c as one 16-byte chunk
    auto store_b_col = [&](const uint4 (&rb)[8], int buf, int c) {
        const unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;
        const int w = c >> 1;
        auto dw = [&](const uint4& v) -> uint32_t { return w == 0 ? v.x : (w == 1 ? v.y : (w == 2 ? v.z : v.w)); };
        uint4 o;
        o.x = __builtin_amdgcn_perm(dw(rb[1]), dw(rb[0]), sel);
        o.y = __builtin_amdgcn_perm(dw(rb[3]), dw(rb[2]), sel);
        o.z = __builtin_amdgcn_perm(dw(rb[5]), dw(rb[4]), sel);
        o.w = __builtin_amdgcn_perm(dw(rb[7]), dw(rb[6]), sel);
        *(uint4*)(lds + ((b_dst0 ^ (16 * c)) + buf * P_STAGE)) = o;
    };

    // One 64-position step on LDS buffer PAR: sub-step 0 also fetches step + 2 into staging set PAR,
    // sub-step 2 writes step + 1 (staging set PAR ^ 1) into LDS buffer PAR ^ 1; then the barrier, and
    // sub-step 3 prefetches its fragments from that buffer.  The last two steps of a workgroup fetch
    // and store tiles nobody uses (reads past the tensors return zero through the descriptors); that
    // keeps the loop body free of branches, which the accumulator registers do not survive well.
    auto run_step = [&](auto par_c, int kk_load) {
        constexpr int PAR = decltype(par_c)::value;
#define PROJ_CHUNK(PH, q, i0, j0, i1, j1, LD)                                                   \
        {                                                                                       \
            constexpr int cur = (PH) & 1, nxt = cur ^ 1, ns = ((PH) + 1) & 3;                   \
            constexpr int pbuf = (PH) == 3 ? (PAR ^ 1) : PAR;                                   \
            PROJ_MMA(cur, i0, j0); PROJ_MMA(cur, i1, j1);                                       \
            LD(nxt, pbuf, ns, (q) >> 1);                                                        \
            if ((PH) == 0) {                                                                    \
                RA[PAR][q] = buf_ld16(rsA, voffA, kk_load * 2 + (q) * rowsA);                   \
                RB[PAR][q] = buf_ld16(rsB, voffB + (q) * (D * 2), kk_load * (D * 2));           \
            }                                                                                   \
            if ((PH) == 2) {                                                                    \
                *(uint4*)(a_dst + (PAR ^ 1) * P_STAGE + (32 * (q)) * PA_PITCH) = RA[PAR ^ 1][q]; \
                store_b_col(RB[PAR ^ 1], PAR ^ 1, q);                                           \
            }                                                                                   \
            PROJ_SB();                                                                          \
        }
#define PROJ_PHASE(PH)                                  \
        PROJ_CHUNK(PH, 0, 0, 0, 0, 1, PROJ_LDA)         \
        PROJ_CHUNK(PH, 1, 1, 0, 1, 1, PROJ_LDB)         \
        PROJ_CHUNK(PH, 2, 0, 2, 1, 2, PROJ_LDA)         \
        PROJ_CHUNK(PH, 3, 0, 3, 1, 3, PROJ_LDB)         \
        PROJ_CHUNK(PH, 4, 2, 0, 2, 1, PROJ_LDA)         \
        PROJ_CHUNK(PH, 5, 3, 0, 3, 1, PROJ_LDB)         \
        PROJ_CHUNK(PH, 6, 2, 2, 3, 2, PROJ_LDA)         \
        PROJ_CHUNK(PH, 7, 2, 3, 3, 3, PROJ_LDB)
        PROJ_PHASE(0)
        PROJ_PHASE(1)
        PROJ_PHASE(2)
        __syncthreads();              // next buffer complete; nobody still reads it
        PROJ_SB();
        PROJ_PHASE(3)
#undef PROJ_PHASE
#undef PROJ_CHUNK
    };

    if (step0 < step1) {
        // prologue: step0 through registers into buffer 0, step0 + 1 into staging set 1
        const int kk0 = step0 * PBK;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            RA[0][q] = buf_ld16(rsA, voffA, kk0 * 2 + q * rowsA);
            RB[0][q] = buf_ld16(rsB, voffB + q * (D * 2), kk0 * (D * 2));
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            RA[1][q] = buf_ld16(rsA, voffA, (kk0 + PBK) * 2 + q * rowsA);
            RB[1][q] = buf_ld16(rsB, voffB + q * (D * 2), (kk0 + PBK) * (D * 2));
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            *(uint4*)(a_dst + (32 * q) * PA_PITCH) = RA[0][q];
            store_b_col(RB[0], 0, q);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) { PROJ_LDA(0, 0, 0, i); PROJ_LDB(0, 0, 0, i); }
        PROJ_SB();
        int step = step0;
        for (; step + 1 < step1; step += 2) {
            run_step(IC<0>{}, (step + 2) * PBK);
            run_step(IC<1>{}, (step + 3) * PBK);
        }
        if (step < step1) run_step(IC<0>{}, (step + 2) * PBK);
    }
#undef PROJ_SB
#undef PROJ_MMA
#undef PROJ_LDA
#undef PROJ_LDB

    // epilogue: fp32 partial sums in (BH, k, d) layout
    float* __restrict__ out = a.out[which] + (long)split * a.split_stride;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = wn * 128 + 32 * j + l32;
        const int bh = bh0 + c / D;
        if (bh >= a.BH) continue;
        float* ob = out + (long)bh * a.k * D + (c % D);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                const int r = m0 + wm * 128 + 32 * i + 8 * (g >> 2) + 4 * half + (g & 3);
                if (r < a.k) ob[(long)r * D] = acc[i][j][g];
            }
        }
    }
}

struct ProjPlan {
    int tilesM, tilesN, splits, steps_per_split, total_steps;
};

static ProjPlan proj_plan(const Problem& p) {
    ProjPlan q;
    q.tilesM = (p.k + PBM - 1) / PBM;
    const int heads_per_tile = PBN / p.d;
    q.tilesN = (p.BH + heads_per_tile - 1) / heads_per_tile;
    q.total_steps = p.n / PBK;
    const int tiles = q.tilesM * q.tilesN * 2;
    int splits = 256 / tiles;                      // one workgroup per compute unit
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
    const uint16_t* St;        // (BH, d, mf) bf16
    const float* zp;           // (BH, mf)
    const float* cp;           // (BH, mf) exponent shifts, same order as zp
    uint16_t* out;
    int n, H, mf, rows_per_wg, wgs_per_head;
    long omega_head_stride;    // 0 if shared
};

template <int D>
struct QueryLds {
    static constexpr int w_pitch = (D + 8) * 2;                  // bytes per omega row
    static __host__ __device__ int s_pitch(int mf) { return (mf + 8) * 2; }
    static __host__ __device__ int w_bytes(int mf) { return mf * w_pitch; }
    static __host__ __device__ int s_bytes(int mf) { return D * s_pitch(mf); }
    static __host__ __device__ int total(int mf, int elu) {
        return (elu ? 0 : w_bytes(mf)) + s_bytes(mf) + mf * 8;
    }
};

// One workgroup = 8 wavefronts sharing the LDS image of omega, S^T and z of one head; each wavefront
// streams 32 query rows at a time.
template <int D, bool ELU>
__global__ __launch_bounds__(512) void query_stream_kernel(QueryArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    using L = QueryLds<D>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int bh = blockIdx.x / a.wgs_per_head;
    const int chunk = blockIdx.x % a.wgs_per_head;
    const int mf = a.mf;
    const int s_pitch = L::s_pitch(mf);
    unsigned char* lw = lds;
    unsigned char* ls = lds + (ELU ? 0 : L::w_bytes(mf));
    float* lz = (float*)(ls + L::s_bytes(mf));
    float* lc = lz + mf;

    // fill the LDS image (16-byte chunks, coalesced)
    if (!ELU) {
        const uint16_t* og = a.omega + (long)(bh % a.H) * a.omega_head_stride;
        constexpr int cpr = D / 8;                      // chunks per row
        for (int c = tid; c < mf * cpr; c += 512) {
            const int r = c / cpr, q = c % cpr;
            *(uint4*)(lw + r * L::w_pitch + 16 * q) = ld16(og + (long)r * D + 8 * q);
        }
    }
    {
        const uint16_t* sg = a.St + (long)bh * D * mf;
        const int cpr = mf / 8;
        for (int c = tid; c < D * cpr; c += 512) {
            const int r = c / cpr, q = c % cpr;
            *(uint4*)(ls + r * s_pitch + 16 * q) = ld16(sg + (long)r * mf + 8 * q);
        }
        const float* zg = a.zp + (long)bh * mf;
        const float* cg = a.cp + (long)bh * mf;
        for (int c = tid; c < mf; c += 512) { lz[c] = zg[c]; lc[c] = cg[c]; }
    }
    __syncthreads();

    const long head_off = (long)bh * a.n * D;
    const int row_begin = chunk * a.rows_per_wg;
    int row_end = row_begin + a.rows_per_wg;
    if (row_end > a.n) row_end = a.n;
    constexpr int KS = D / 16;      // reduction steps over d
    constexpr int TT = D / 32;      // 32-row tiles of N^T
    constexpr float LOG2E = 1.4426950408889634f;

    for (int row0 = row_begin + 32 * wave; row0 < row_end; row0 += 32 * 8) {
        // B operand of the first contraction: this lane's query row, 8 consecutive d per step
        int qrow = row0 + l32;
        const bool valid = qrow < a.n;
        if (!valid) qrow = a.n - 1;
        const uint16_t* qg = a.Q + head_off + (long)qrow * D + 8 * half;
        uint4 qf[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = ld16(qg + 16 * s);

        floatx16 accN[TT];
#pragma unroll
        for (int t = 0; t < TT; ++t) accN[t] = zero16();
        float den = 0.f;

        if (ELU) {
            // P = elu(q)+1 straight in operand order; features are the d coordinates
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const uint32_t w[4] = {qf[s].x, qf[s].y, qf[s].z, qf[s].w};
                uint32_t pk[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x0 = bf16_to_f32((uint16_t)(w[e] & 0xffffu));
                    const float x1 = bf16_to_f32((uint16_t)(w[e] >> 16));
                    const float p0 = x0 > 0.f ? x0 + 1.f : __expf(x0);
                    const float p1 = x1 > 0.f ? x1 + 1.f : __expf(x1);
                    pk[e] = pack_bf16(p0, p1);
                    const int f = 16 * s + 8 * half + 2 * e;
                    den = fmaf(p0, lz[f], den);
                    den = fmaf(p1, lz[f + 1], den);
                }
                const uint4 pb = {pk[0], pk[1], pk[2], pk[3]};
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    const uint4 sa = *(const uint4*)(ls + (32 * t + l32) * s_pitch + 32 * s + 16 * half);
                    accN[t] = mfma32(sa, pb, accN[t]);
                }
            }
        } else {
            float mu = -INFINITY;     // running row maximum (same value in lanes l and l^32)
            for (int ft = 0; ft < mf / 32; ++ft) {
                // accumulator starts at the key side's per-feature shift: u_j + c_j is the true
                // log-weight, and the add costs nothing
                floatx16 u;
                {
                    const float4* ct = (const float4*)(lc + 32 * ft + 16 * half);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 v = ct[q];
                        u[4 * q] = v.x; u[4 * q + 1] = v.y; u[4 * q + 2] = v.z; u[4 * q + 3] = v.w;
                    }
                }
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const uint4 wa = *(const uint4*)(lw + (32 * ft + l32) * L::w_pitch + 32 * s + 16 * half);
                    u = mfma32(wa, qf[s], u);
                }
                float tmax = fmaxf(fmaxf(u[0], u[1]), u[2]);
#pragma unroll
                for (int g = 3; g < 15; g += 2) tmax = fmaxf(fmaxf(tmax, u[g]), u[g + 1]);
                tmax = fmaxf(tmax, u[15]);
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
                if (tmax > mu) {
                    const float sc = fast_exp2((mu - tmax) * LOG2E);     // 0 on the first tile
                    mu = tmax;
                    den *= sc;
#pragma unroll
                    for (int t = 0; t < TT; ++t)
#pragma unroll
                        for (int g = 0; g < 16; ++g) accN[t][g] *= sc;
                }
                const float nshift = -mu * LOG2E;
                const float4* zt = (const float4*)(lz + 32 * ft + 16 * half);
                uint32_t pk[8];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 zv = zt[q];
                    const float p0 = fast_exp2(fmaf(u[4 * q], LOG2E, nshift));
                    const float p1 = fast_exp2(fmaf(u[4 * q + 1], LOG2E, nshift));
                    const float p2 = fast_exp2(fmaf(u[4 * q + 2], LOG2E, nshift));
                    const float p3 = fast_exp2(fmaf(u[4 * q + 3], LOG2E, nshift));
                    pk[2 * q] = pack_bf16(p0, p1);
                    pk[2 * q + 1] = pack_bf16(p2, p3);
                    den = fmaf(p0, zv.x, den);
                    den = fmaf(p1, zv.y, den);
                    den = fmaf(p2, zv.z, den);
                    den = fmaf(p3, zv.w, den);
                }
                const uint4 pb0 = {pk[0], pk[1], pk[2], pk[3]};
                const uint4 pb1 = {pk[4], pk[5], pk[6], pk[7]};
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    const unsigned char* sp = ls + (32 * t + l32) * s_pitch + 64 * ft + 16 * half;
                    accN[t] = mfma32(*(const uint4*)sp, pb0, accN[t]);
                    accN[t] = mfma32(*(const uint4*)(sp + 32), pb1, accN[t]);
                }
            }
        }
        den += __shfl_xor(den, 32, 64);
        const float inv = 1.f / den;
        if (valid) {
            uint16_t* og = a.out + head_off + (long)qrow * D;
#pragma unroll
            for (int t = 0; t < TT; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 v;
                    v.x = pack_bf16(accN[t][4 * q] * inv, accN[t][4 * q + 1] * inv);
                    v.y = pack_bf16(accN[t][4 * q + 2] * inv, accN[t][4 * q + 3] * inv);
                    *(uint2*)(og + 32 * t + 8 * q + 4 * half) = v;
                }
        }
    }
}

// ===========================================================================
// Host side
// ===========================================================================
static int query_lds_bytes(const Problem& p) {
    return p.d == 64 ? QueryLds<64>::total(p.mf, p.elu) : QueryLds<128>::total(p.mf, p.elu);
}

bool fast_supported(const Problem& p, int bwd) {
    if (bwd) return fast_bwd_supported(p);
    if (!p.bf16) return false;
    if (p.d != 64 && p.d != 128) return false;
    if (p.n % PBK != 0) return false;
    if (p.mf % 32 != 0) return false;
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
    size_t partial, Kimg, Vimg, nrm, Spart, zpart, cpart, St, zp, cp, total;    // byte offsets
    size_t split_stride;              // floats between the partial results of consecutive splits
};

static FastWs fast_ws_layout(const Problem& p) {
    FastWs W{};
    const CtxLayout L = ctx_layout(p);
    const ProjPlan q = proj_plan(p);
    const KeyStatePlan ks = key_state_plan(p);
    const size_t BH = (size_t)p.BH;
    size_t o = 0;
    W.split_stride = L.S;             // K' and V' segments of ctx, back to back
    W.partial = o; o += round_up((q.splits > 1 ? (size_t)q.splits : 0) * W.split_stride * 4, 256);
    W.Kimg = o;    o += round_up(p.elu ? 0 : 3 * BH * ks.kpad * p.d * 2, 256);
    W.Vimg = o;    o += round_up(2 * BH * (ks.kpad / 2) * p.d * 4, 256);
    W.nrm = o;     o += round_up(BH * ks.kpad * 4, 256);
    W.Spart = o;   o += round_up(BH * ks.KR * p.mf * p.d * 4, 256);
    W.zpart = o;   o += round_up(BH * ks.KR * p.mf * 4, 256);
    W.cpart = o;   o += round_up(BH * ks.KR * p.mf * 4, 256);
    W.St = o;      o += round_up(BH * p.d * p.mf * 2, 256);
    W.zp = o;      o += round_up(BH * p.mf * 4, 256);
    W.cp = o;      o += round_up(BH * p.mf * 4, 256);
    W.total = o;
    return W;
}

size_t fast_ws_bytes(const Problem& p, int bwd) {
    return bwd ? fast_bwd_ws_bytes(p) : fast_ws_layout(p).total;
}

template <int D, bool ELU>
static flurka_status launch_query(const Problem& p, const QueryArgs& qa, int grid, int ldsb, hipStream_t s) {
    auto kern = query_stream_kernel<D, ELU>;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ldsb) != hipSuccess)
        return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), ldsb, s, qa);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

flurka_status fast_forward(const Problem& p, const FwdArgs& a, hipStream_t s) {
    const CtxLayout L = ctx_layout(p);
    const FastWs W = fast_ws_layout(p);
    unsigned char* wsb = (unsigned char*)a.ws;
    flurka_status st;
    int proj_splits = 1;
    {
        StageScope sc(s, STAGE_PROJECT);
        const ProjPlan q = proj_plan(p);
        ProjArgs pa{};
        pa.EF[0] = (const uint16_t*)a.E; pa.EF[1] = (const uint16_t*)a.F;
        pa.X[0] = (const uint16_t*)a.K;  pa.X[1] = (const uint16_t*)a.V;
        float* base = q.splits > 1 ? (float*)(wsb + W.partial) : a.ctx;
        pa.out[0] = base + L.Kp;
        pa.out[1] = base + L.Vp;
        pa.split_stride = (long)W.split_stride;
        pa.n = p.n; pa.d = p.d; pa.k = p.k; pa.BH = p.BH;
        pa.tilesM = q.tilesM; pa.tilesN = q.tilesN; pa.splits = q.splits;
        pa.steps_per_split = q.steps_per_split; pa.total_steps = q.total_steps;
        const void* kern = p.d == 64 ? (const void*)proj_mfma_kernel<64> : (const void*)proj_mfma_kernel<128>;
        if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS) != hipSuccess)
            return FLURKA_ERR_LAUNCH;
        const int grid = q.tilesM * q.tilesN * 2 * q.splits;
        if (p.d == 64) hipLaunchKernelGGL(proj_mfma_kernel<64>, dim3(grid), dim3(256), P_LDS, s, pa);
        else           hipLaunchKernelGGL(proj_mfma_kernel<128>, dim3(grid), dim3(256), P_LDS, s, pa);
        FLURKA_CHECK_LAUNCH();
        proj_splits = q.splits;
    }
    {
        StageScope sc(s, STAGE_KEY_STATE);
        KeyStateBuffers kb{};
        kb.Kimg = (uint16_t*)(wsb + W.Kimg); kb.Vimg = (uint32_t*)(wsb + W.Vimg); kb.nrm = (float*)(wsb + W.nrm);
        kb.Spart = (float*)(wsb + W.Spart); kb.zpart = (float*)(wsb + W.zpart); kb.cpart = (float*)(wsb + W.cpart);
        kb.St = (uint16_t*)(wsb + W.St); kb.zp = (float*)(wsb + W.zp); kb.cp = (float*)(wsb + W.cp);
        const float* partials = proj_splits > 1 ? (const float*)(wsb + W.partial) : a.ctx;
        st = fast_key_state(p, a.omega, a.ctx, partials, (long)W.split_stride, proj_splits, kb, s);
        if (st != FLURKA_OK) return st;
    }
    {
        StageScope sc(s, STAGE_QUERY);
        QueryArgs qa{};
        qa.Q = (const uint16_t*)a.Q;
        qa.omega = (const uint16_t*)a.omega;
        qa.St = (const uint16_t*)(wsb + W.St);
        qa.zp = (const float*)(wsb + W.zp);
        qa.cp = (const float*)(wsb + W.cp);
        qa.out = (uint16_t*)a.out;
        qa.n = p.n; qa.H = p.H; qa.mf = p.mf;
        qa.omega_head_stride = p.omega_per_head ? (long)p.m * p.d : 0;
        // about two workgroups per compute unit, each a multiple of 256 rows (8 wavefronts x 32)
        int wgs_per_head = (512 + p.BH - 1) / p.BH;
        int rows = (p.n + wgs_per_head - 1) / wgs_per_head;
        rows = (rows + 255) / 256 * 256;
        wgs_per_head = (p.n + rows - 1) / rows;
        qa.rows_per_wg = rows; qa.wgs_per_head = wgs_per_head;
        const int grid = p.BH * wgs_per_head;
        const int ldsb = query_lds_bytes(p);
        if (p.d == 64)
            st = p.elu ? launch_query<64, true>(p, qa, grid, ldsb, s) : launch_query<64, false>(p, qa, grid, ldsb, s);
        else
            st = p.elu ? launch_query<128, true>(p, qa, grid, ldsb, s) : launch_query<128, false>(p, qa, grid, ldsb, s);
        if (st != FLURKA_OK) return st;
    }
    return FLURKA_OK;
}


}  // namespace flurka
