// One 256 x 256 x 64 bf16 MFMA GEMM main loop for gfx950, shared by the three large contractions
// of FLuRKA attention.  What differs between them (where the operands live, how a reduction step
// maps to addresses, where the result goes) is supplied by a policy type:
//
//   ProjPolicy<D>   K' = E K, V' = F V          A = E rows, B = X (positions x columns, read out of LDS
//                                               with transposing loads), fp32 split partials
//   GradXPolicy<D>  dK = E^T dK', dV = F^T dV'  A = (dK')^T image rows, B = E (same path as X above),
//                                               bf16 result stored transposed into (B,H,n,d)
//   GradEPolicy<D>  dE = sum_bh dK' K^T         A = dK' image rows, B = K rows (both contiguous along
//                                               the reduction), fp32 split partials
//
// Structure (one wavefront per SIMD, 4 per workgroup, wave tile 128 x 128 = 4 x 4 MFMA tiles, so all
// latency hiding happens inside one instruction stream): a 64-deep step is four 16-deep sub-steps of
// 16 MFMAs, i.e. 32 chunks of "2 MFMAs + one LDS fragment read".  While sub-step s multiplies, the
// fragments of sub-step s+1 are read from LDS into the other fragment register set.  Global data runs
// two steps ahead through ONE set of 16 staging registers reused in place: register j requests its
// part of the tile in even chunk 2j and stores it to LDS 25 chunks later (an odd chunk), after which
// it is free for its next request; so requests and LDS stores are spread evenly over the step instead
// of arriving in bursts that fill the address FIFOs.  One barrier per step, before sub-step 3, which
// already prefetches fragments from the other buffer.  sched_barrier(0) after each chunk pins this
// order.  The last two steps fetch and store tiles nobody uses; that keeps the loop body free of
// branches, which the 256 accumulator registers do not survive well.
#pragma once

#include "flurka_mfma.h"

namespace flurka {

constexpr int GBM = 256, GBN = 256, GBK = 64;
constexpr int GA_PITCH = 144;                       // bytes per LDS row of a row-major tile (128 + 16)
constexpr int GA_STAGE = GBM * GA_PITCH;            // 36,864
constexpr int GB_PITCH_T = GBN * 2 + 64;            // row of a [position][column] tile: 4 consecutive rows
                                                    // fall into the 4 quarters of the LDS banks
constexpr int GB_STAGE_T = GBK * GB_PITCH_T;        // 36,864
constexpr int GB_STAGE_D = GBN * GA_PITCH;          // direct tile: like A
constexpr int G_STAGE = GA_STAGE + GB_STAGE_D;      // 73,728 (both layouts of B take the same room)
static_assert(GB_STAGE_T <= GB_STAGE_D, "B stage");
constexpr int G_LDS_STAGES = 2 * G_STAGE;           // 147,456
constexpr int G_LDS_EPI = 4 * 4096;                 // per wavefront: a 32 x 64 bf16 tile on its way out
constexpr int G_LDS = G_LDS_STAGES + G_LDS_EPI;     // 163,840: all of a compute unit's LDS
constexpr int G_OOB = 0x7fffff00;                   // per-thread byte offset past any descriptor range

// fp32 partial results of a split reduction are kept tile by tile in the order the accumulators
// hold them, so that every store is 16 bytes per lane and 1 KiB per wavefront, with no bounds to check
// (whole tiles are allocated).  Tile t of (which, split, column tile, row tile) starts at
// partial_tile_index(...) * G_TILE_ELEMS floats; inside it element (r, c) of the 256 x 256 tile sits at
// partial_elem_offset(r, c): [wavefront 2*(r/128) + c/128][i = r/32 % 4][j = c/32 % 4][q = r/8 % 4]
// [lane = 32*(r/4 % 2) + c%32][e = r%4].
constexpr int G_TILE_ELEMS = 256 * 256;
__host__ __device__ inline long partial_tile_index(int which, int split, int tn, int tm, int splits, int tilesN,
                                                   int tilesM) {
    return (((long)which * splits + split) * tilesN + tn) * tilesM + tm;
}
__host__ __device__ inline int partial_elem_offset(int r, int c) {
    const int wave = 2 * (r >> 7) + (c >> 7), i = (r >> 5) & 3, j = (c >> 5) & 3, q = (r >> 3) & 3;
    const int lane = 32 * ((r >> 2) & 1) + (c & 31), e = r & 3;
    return ((((wave * 4 + i) * 4 + j) * 4 + q) * 64 + lane) * 4 + e;
}

struct GemmParams {
    const uint16_t* A[2];
    const uint16_t* B[2];
    void* C[2];              // result tensors (policies that store final results); C[0] = partial buffer
                             // for policies with PARTIAL_TILES
    int tilesM, tilesN, splits, steps_per_split, total_steps;
    int n, d, k, BH, kp;     // problem sizes the policies need (kp: padded k of an image)
    int dm, tiles_per_batch; // model width and 256-column tiles per batch (policies of the paper-order path)
};

template <int N>
struct IC { static constexpr int value = N; };

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16-byte load through a buffer descriptor: per-thread byte offset + wave-uniform byte offset;
// addresses past the descriptor's range read as zero
__device__ __forceinline__ uint4 buf_ld16(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

typedef short gemm_short4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 gemm_read_tr16(const unsigned char* p) {
    const gemm_short4 v =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((gemm_short4 __attribute__((address_space(3)))*)p);
    return __builtin_bit_cast(uint2, v);
}

// ids handed to workgroups (SHARE_B pads the (split, column tile, which) index to a multiple of 8)
template <class Pol>
__host__ __device__ inline int gemm_item_count(const GemmParams& g) {
    const int outer = g.splits * g.tilesN * 2;
    return Pol::SHARE_B ? 8 * g.tilesM * ((outer + 7) / 8) : g.tilesM * outer;
}

// STREAM: a workgroup may take several work items (launched with fewer workgroups than items); the
// one-item form keeps the step bookkeeping out of the long reductions, where it costs a few percent.
// `block` of `nblocks`: this workgroup's place among the workgroups that share the items
// item_lo .. item_hi - 1 of this GEMM (the whole grid and all items, or one part of a grid that runs two
// GEMMs side by side; item_lo a multiple of 8, item_hi at most the item count).
template <class Pol, bool STREAM>
__device__ __forceinline__ void gemm_mfma_body(const GemmParams& g, const int block, const int nblocks,
                                               unsigned char* const lds, const int item_lo, const int item_hi) {
    constexpr bool BT = Pol::B_TRANSPOSE;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int half = lane >> 5, l32 = lane & 31;

    // Work items = (split, row tile, column tile, which).  A workgroup takes items block,
    // block + nblocks, ... (nblocks is a multiple of 8 whenever there is more than one item per
    // workgroup, so a workgroup's items all run on one XCD = id mod 8) and runs their reduction steps as
    // ONE stream: the requests issued during the last two steps of an item already fetch the first two
    // steps of the next one, so only the first item of a workgroup pays for an empty pipeline.
    // Order of ids:
    //   split-major (projection): consecutive ids walk the splits first, so with a split count that is a
    //     multiple of 8 every XCD keeps to its own reduction range of both operands;
    //   SHARE_B (gradient GEMMs, whose B operand is the large one): id mod 8 is the low part of the
    //     (split, column tile, which) index and the row tiles follow, so all row tiles that read one B
    //     tile run on the same XCD at about the same time and that tile leaves HBM once.
    struct Item { int split, tm, tn, which, step0, step1, send; bool valid; };
    auto decode = [&](int id) -> Item {
        Item it;
        it.valid = id < item_hi;
        if (!it.valid) id = 0;
        if constexpr (Pol::SHARE_B) {
            const int xcd = id & 7; id >>= 3;
            it.tm = id % g.tilesM;    id /= g.tilesM;
            int u = 8 * id + xcd;                                     // (split, column tile, which)
            it.split = u % g.splits;  u /= g.splits;
            it.tn = u % g.tilesN;     u /= g.tilesN;
            it.which = u;
            if (u > 1) { it.valid = false; it.which = 0; }            // only past the last real item
        } else {
            it.split = id % g.splits; id /= g.splits;
            it.tm = id % g.tilesM;    id /= g.tilesM;
            it.tn = id % g.tilesN;    id /= g.tilesN;
            it.which = id;
        }
        it.step0 = it.split * g.steps_per_split;
        it.step1 = it.step0 + g.steps_per_split;
        if (it.step1 > g.total_steps) it.step1 = g.total_steps;
        if (!it.valid) it.step1 = it.step0;                           // nothing of it is real
        it.send = it.step0 + ((it.step1 - it.step0 + 1) & ~1);        // steps run in pairs
        return it;
    };
    int item_id = item_lo + block;
    Item cur = decode(item_id), nxt = decode(STREAM ? item_id + nblocks : item_hi);
    typename Pol::Ctx pc = Pol::make(g, cur.which, cur.tm * GBM, cur.tn * GBN, tid);
    typename Pol::Ctx pn = Pol::make(g, nxt.which, nxt.tm * GBM, nxt.tn * GBN, tid);

    // LDS addresses of this thread's writes and of this lane's fragment reads (per buffer: + G_STAGE)
    unsigned char* const a_dst = lds + (tid >> 3) * GA_PITCH + 16 * (tid & 7);                    // + 32*q rows
    const unsigned char* const fa_src = lds + (wm * 128 + l32) * GA_PITCH + 16 * half;           // + 32*i rows, + 32*s
    // B given as [position][column] ("transposed" with respect to what the MFMA wants): the tile goes
    // to LDS as loaded, thread = (8 positions b_kg, 8 columns b_cg), and the fragments come out through
    // ds_read_b64_tr_b16: in each group of 16 lanes, lane s points at 4 columns of row s/4 of a
    // 4 x 16 block and receives one column of its 4 rows; two such reads are the 8 reduction slots.
    const int b_cg = tid & 31, b_kg = tid >> 5;
    unsigned char* const bt_dst = lds + GA_STAGE + (8 * b_kg) * GB_PITCH_T + 16 * b_cg;          // + q rows
    unsigned char* const bd_dst = lds + GA_STAGE + (tid >> 3) * GA_PITCH + 16 * (tid & 7);       // direct B
    const unsigned char* fb_src[4];
    if (BT) {
        const int s16 = lane & 15;
        const int row = 8 * half + (s16 >> 2), colb = 2 * (wn * 128 + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3));
#pragma unroll
        for (int j = 0; j < 4; ++j) fb_src[j] = lds + GA_STAGE + row * GB_PITCH_T + colb + 64 * j;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) fb_src[j] = lds + GA_STAGE + (wn * 128 + 32 * j + l32) * GA_PITCH + 16 * half;
    }

    uint4 RA[8], RB[8];
    uint4 FA[2][4], FB[2][4];
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = zero16();

#define G_SB() __builtin_amdgcn_sched_barrier(0)
#define G_MMA(set, i, j) acc[i][j] = mfma32(FA[set][i], FB[set][j], acc[i][j])
#define G_LDA(set, buf, s, i) \
    FA[set][i] = *(const uint4*)(fa_src + (buf) * G_STAGE + (32 * (i)) * GA_PITCH + 32 * (s))
#define G_LDB(set, buf, s, j)                                                                         \
    if (BT) {                                                                                         \
        const unsigned char* bp_ = fb_src[j] + (buf) * G_STAGE + (16 * (s)) * GB_PITCH_T;             \
        const uint2 lo_ = gemm_read_tr16(bp_), hi_ = gemm_read_tr16(bp_ + 4 * GB_PITCH_T);            \
        FB[set][j] = make_uint4(lo_.x, lo_.y, hi_.x, hi_.y);                                          \
    } else {                                                                                          \
        FB[set][j] = *(const uint4*)(fb_src[j] + (buf) * G_STAGE + 32 * (s));                         \
    }

    // staging register q of A / B into LDS buffer `buf`
    auto store_a = [&](int buf, int q) { *(uint4*)(a_dst + buf * G_STAGE + (32 * q) * GA_PITCH) = RA[q]; };
    auto store_b = [&](int buf, int q) {
        if (BT) *(uint4*)(bt_dst + buf * G_STAGE + q * GB_PITCH_T) = RB[q];
        else    *(uint4*)(bd_dst + buf * G_STAGE + (32 * q) * GA_PITCH) = RB[q];
    };

    auto run_step = [&](auto par_c, int step_load) {
        constexpr int PAR = decltype(par_c)::value;
        // where the step two ahead comes from: this item, its zero step (odd counts), or the next item
        const bool in_cur = !STREAM || step_load < cur.send;
        const int sl = in_cur ? step_load : nxt.step0 + (step_load - cur.send);
        const bool real = in_cur ? step_load < cur.step1 : sl < nxt.step1;
        const typename Pol::Ctx& sc = in_cur ? pc : pn;
        const int sA = Pol::a_soff(sc, sl), sB = Pol::b_soff(sc, sl);
        const __amdgpu_buffer_rsrc_t rsA = sc.rsA, rsB = sc.rsB;
        const int voffA = sc.voffA, aq = sc.a_qstride, bq = sc.b_qstride;
        const int vB = real ? sc.voffB : G_OOB;                 // past the range: B reads as zero
        // B_ROW_LIMIT: rows of B are reduction positions of which only b_rows exist (a ragged last
        // step); this thread's row q of the step exists if q < b_left
        int b_left = 8;
        if constexpr (Pol::B_ROW_LIMIT) b_left = sc.b_rows - (sl * GBK + 8 * b_kg);
#define G_CHUNK(PH, q, i0, j0, i1, j1, LD)                                                      \
        {                                                                                       \
            constexpr int cur = (PH) & 1, nxt = cur ^ 1, ns = ((PH) + 1) & 3;                   \
            constexpr int pbuf = (PH) == 3 ? (PAR ^ 1) : PAR;                                   \
            G_MMA(cur, i0, j0); G_MMA(cur, i1, j1);                                             \
            LD(nxt, pbuf, ns, (q) >> 1);                                                        \
            constexpr int pos = 8 * (PH) + (q);      /* 0..31 within the step */                \
            /* even chunk 2j: staging register j (A and B alternate) requests its part of the   */ \
            /* tile two steps ahead; 25 chunks later (odd chunk) it is stored to LDS: chunks     */ \
            /* 25..31 store into this step's own buffer, which nobody reads after the barrier,   */ \
            /* chunks 1..23 of the next step finish the other buffer before that step's barrier  */ \
            if ((pos & 1) == 0) {                                                               \
                constexpr int j = pos / 2;                                                      \
                if (j & 1) RB[j / 2] = buf_ld16(rsB, (!Pol::B_ROW_LIMIT || j / 2 < b_left) ? vB : G_OOB, \
                                                sB + (j / 2) * bq);                             \
                else       RA[j / 2] = buf_ld16(rsA, voffA, sA + (j / 2) * aq);                 \
            } else {                                                                            \
                constexpr int j = ((pos + 7) & 31) / 2;                                         \
                constexpr int wbuf = pos >= 25 ? PAR : (PAR ^ 1);                               \
                if (j & 1) store_b(wbuf, j / 2);                                                \
                else       store_a(wbuf, j / 2);                                                \
            }                                                                                   \
            G_SB();                                                                             \
        }
#define G_PHASE(PH)                               \
        G_CHUNK(PH, 0, 0, 0, 0, 1, G_LDA)         \
        G_CHUNK(PH, 1, 1, 0, 1, 1, G_LDB)         \
        G_CHUNK(PH, 2, 0, 2, 1, 2, G_LDA)         \
        G_CHUNK(PH, 3, 0, 3, 1, 3, G_LDB)         \
        G_CHUNK(PH, 4, 2, 0, 2, 1, G_LDA)         \
        G_CHUNK(PH, 5, 3, 0, 3, 1, G_LDB)         \
        G_CHUNK(PH, 6, 2, 2, 3, 2, G_LDA)         \
        G_CHUNK(PH, 7, 2, 3, 3, 3, G_LDB)
        G_PHASE(0)
        G_PHASE(1)
        G_PHASE(2)
        __syncthreads();              // next buffer complete; nobody still reads it
        G_SB();
        G_PHASE(3)
#undef G_PHASE
#undef G_CHUNK
    };

    auto epilogue = [&](const Item& it) {
        // this lane holds, for every 32 x 32 tile (i, j), column 32*j + l32 and rows
        // 32*i + 8*q + 4*half + {0..3}, q = 0..3
        if constexpr (Pol::PARTIAL_TILES) {
            float* tp = (float*)g.C[0] +
                        partial_tile_index(it.which, it.split, it.tn, it.tm, g.splits, g.tilesN, g.tilesM) * G_TILE_ELEMS +
                        (long)wave * (16 * 4 * 256) + lane * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float4 v;
                        v.x = acc[i][j][4 * q]; v.y = acc[i][j][4 * q + 1]; v.z = acc[i][j][4 * q + 2]; v.w = acc[i][j][4 * q + 3];
                        *(float4*)(tp + ((i * 4 + j) * 4 + q) * 256) = v;
                    }
        } else if constexpr (Pol::TRANSPOSED_STORE) {
            // The result leaves transposed: element (row r, column c) goes to C[c][r], 64 consecutive r
            // being 128 contiguous bytes.  Each wavefront turns its accumulators, 64 rows x 32 columns at
            // a time, through a private 4 KiB LDS area ([column][row], 16-byte chunk k of column c at
            // chunk position k ^ ((c >> 1) & 7)): 8-byte pieces in, 16-byte chunks out, so that one
            // store instruction covers 8 columns x 128 bytes instead of 64 separate 16-byte pieces.
            // (The stage buffers already hold the next item's first steps and are not touched.)
            unsigned char* const tr = lds + G_LDS_STAGES + wave * 4096;
            const int m0 = it.tm * GBM, n0 = it.tn * GBN;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int ip = 0; ip < 2; ++ip) {
#pragma unroll
                    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const floatx16& t = acc[2 * ip + ii][j];
                            uint2 v;
                            v.x = pack_bf16(t[4 * q], t[4 * q + 1]);
                            v.y = pack_bf16(t[4 * q + 2], t[4 * q + 3]);
                            *(uint2*)(tr + l32 * 128 + 16 * ((4 * ii + q) ^ ((l32 >> 1) & 7)) + 8 * half) = v;
                        }
                    const int r0 = m0 + wm * 128 + 64 * ip;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int c = 8 * u + (lane >> 3), k = lane & 7;
                        const uint4 v = *(const uint4*)(tr + c * 128 + 16 * (k ^ ((c >> 1) & 7)));
                        Pol::store_rows(g, it.which, r0, n0 + wn * 128 + 32 * j + c, k, v);
                    }
                }
        } else {
            // groups q and q + 1 are handed over together so that a policy may join the two halves of a
            // wavefront into 8 consecutive rows per lane
            const int m0 = it.tm * GBM, n0 = it.tn * GBN;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = n0 + wn * 128 + 32 * j + l32;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int q = 0; q < 4; q += 2) {
                        const int row = m0 + wm * 128 + 32 * i + 8 * q;
                        const float ev[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                        const float od[4] = {acc[i][j][4 * q + 4], acc[i][j][4 * q + 5], acc[i][j][4 * q + 6], acc[i][j][4 * q + 7]};
                        Pol::store_groups(g, pc, it.which, it.split, row, half, col, ev, od);
                    }
            }
        }
    };

    if (cur.valid && cur.step0 < cur.step1) {
        // prologue (first item only): step0 through the staging registers into buffer 0; step0 + 1
        // requested, its first four registers (the ones the steady state stores in chunks 25..31) stored
        // into buffer 1
        {
            const int sA = Pol::a_soff(pc, cur.step0), sB = Pol::b_soff(pc, cur.step0);
            int b_left = 8;
            if constexpr (Pol::B_ROW_LIMIT) b_left = pc.b_rows - (cur.step0 * GBK + 8 * b_kg);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                RA[q] = buf_ld16(pc.rsA, pc.voffA, sA + q * pc.a_qstride);
                RB[q] = buf_ld16(pc.rsB, q < b_left ? pc.voffB : G_OOB, sB + q * pc.b_qstride);
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) { store_a(0, q); store_b(0, q); }
        {
            const int sA = Pol::a_soff(pc, cur.step0 + 1), sB = Pol::b_soff(pc, cur.step0 + 1);
            const int vB = cur.step0 + 1 < cur.step1 ? pc.voffB : G_OOB;
            int b_left = 8;
            if constexpr (Pol::B_ROW_LIMIT) b_left = pc.b_rows - ((cur.step0 + 1) * GBK + 8 * b_kg);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                RA[q] = buf_ld16(pc.rsA, pc.voffA, sA + q * pc.a_qstride);
                RB[q] = buf_ld16(pc.rsB, q < b_left ? vB : G_OOB, sB + q * pc.b_qstride);
            }
        }
        store_a(1, 0); store_b(1, 0); store_a(1, 1); store_b(1, 1);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) { G_LDA(0, 0, 0, i); G_LDB(0, 0, 0, i); }
        G_SB();
        for (;;) {
            // steps always run in pairs (the two LDS buffers are compile-time roles); an odd count is
            // completed by a step whose B tile reads as zero and so adds nothing
            for (int step = cur.step0; step < cur.send; step += 2) {
                run_step(IC<0>{}, step + 2);
                run_step(IC<1>{}, step + 3);
            }
            epilogue(cur);
            if (!STREAM || !nxt.valid) break;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = zero16();
            item_id += nblocks;
            cur = nxt;
            pc = pn;
            nxt = decode(item_id + nblocks);
            pn = Pol::make(g, nxt.which, nxt.tm * GBM, nxt.tn * GBN, tid);
        }
    }
#undef G_SB
#undef G_MMA
#undef G_LDA
#undef G_LDB
}

template <class Pol, bool STREAM>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmParams g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    gemm_mfma_body<Pol, STREAM>(g, (int)blockIdx.x, (int)gridDim.x, lds, 0, gemm_item_count<Pol>(g));
}

// Two independent GEMMs in one launch, a few long items (first) and many short ones (second).  Each
// alone would leave compute units idle or pay its ramp-up and tail on its own.  The grid is one resident
// round: workgroups 0 .. blocks_a - 1 stream the first GEMM's items and then the last
// items_b - main_b items of the second; the others stream items 0 .. main_b - 1 of the second.  The
// host picks blocks_a and main_b so that both kinds of workgroup finish together.  blocks_a and main_b
// are multiples of 8, so id mod 8 names the XCD in every part.
struct PairPlan {
    int blocks_a;      // workgroups that start with the first GEMM
    int main_b;        // items of the second GEMM that the other workgroups share
    int items_a, items_b;
};

template <class PolA, class PolB>
__global__ __launch_bounds__(256) void gemm_mfma_pair_kernel(GemmParams ga, GemmParams gb, PairPlan pl) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int b = (int)blockIdx.x;
    if (b < pl.blocks_a) {
        gemm_mfma_body<PolA, true>(ga, b, pl.blocks_a, lds, 0, pl.items_a);
        if (pl.main_b < pl.items_b) {
            __syncthreads();           // every wavefront is done with the stage buffers of the first part
            gemm_mfma_body<PolB, true>(gb, b, pl.blocks_a, lds, pl.main_b, pl.items_b);
        }
    } else {
        gemm_mfma_body<PolB, true>(gb, b - pl.blocks_a, (int)gridDim.x - pl.blocks_a, lds, 0, pl.main_b);
    }
}

// ---------------------------------------------------------------------------
// Policies.  Common contract:
//   Ctx make(g, which, m0, n0, tid)   descriptors and this thread's byte offsets
//   a_soff / b_soff (ctx, step)       wave-uniform byte offset of a reduction step
//   a_qstride / b_qstride             byte offset between the 8 loads (q = 0..7) of one step
//   store_groups(..., row, half, col, ev, od)   this lane's rows row + 4*half + {0..3} (ev) and
//                                     row + 8 + 4*half + {0..3} (od) of column col
//   store_rows(..., r0, col, k, v)    (TRANSPOSED_STORE) 8 consecutive rows r0 + 8k.. of column col
// A tile: thread loads 16-byte chunk (tid & 7) of rows (tid >> 3) + 32*q.
// B transposed: thread loads columns 8*(tid & 31).. of positions 8*(tid >> 5) + q.
// B direct: like A, rows being the columns of the result.
// ---------------------------------------------------------------------------
struct PolicyCtxBase {
    __amdgpu_buffer_rsrc_t rsA, rsB;
    int voffA, voffB, a_qstride, b_qstride;
    int b_rows;          // B_ROW_LIMIT policies: number of reduction positions that exist
};

// K' = E K: rows = k projected slots, columns = (head, t), reduction = sequence positions.
template <int D>
struct ProjPolicy {
    static constexpr bool B_TRANSPOSE = true;
    static constexpr bool PARTIAL_TILES = true;
    static constexpr bool TRANSPOSED_STORE = false;
    static constexpr bool SHARE_B = false;
    static constexpr bool B_ROW_LIMIT = true; 
    struct Ctx : PolicyCtxBase { int bh0; };
    static __device__ __forceinline__ Ctx make(const GemmParams& g, int which, int m0, int n0, int tid) {
        Ctx c;
        constexpr int hpt = GBN / D;
        c.bh0 = (n0 / GBN) * hpt;
        int tile_heads = g.BH - c.bh0;
        if (tile_heads > hpt) tile_heads = hpt;
        c.rsA = make_rsrc(g.A[which], (unsigned)g.k * (unsigned)g.n * 2u);
        c.rsB = make_rsrc(g.B[which] + (long)c.bh0 * g.n * D, (unsigned)tile_heads * (unsigned)g.n * (unsigned)(D * 2));
        c.voffA = ((m0 + (tid >> 3)) * g.n + 8 * (tid & 7)) * 2;
        c.a_qstride = 64 * g.n;
        const int b_col = 8 * (tid & 31), b_kg = tid >> 5;
        c.voffB = (((b_col / D) * g.n + 8 * b_kg) * D + (b_col % D)) * 2;
        c.b_qstride = D * 2;
        c.b_rows = g.n;
        return c;
    }
    static __device__ __forceinline__ int a_soff(const Ctx&, int step) { return step * (GBK * 2); }
    static __device__ __forceinline__ int b_soff(const Ctx&, int step) { return step * (GBK * D * 2); }
};

// Paper-order path, first product: Y = E X for the model-wide layer input X (B, n, dm) before any
// per-head transform (Eq. 2: the sequence projection comes first).  Rows = k projected slots, columns =
// (batch, model coordinate), reduction = sequence positions; like ProjPolicy with row stride dm.
struct ProjWidePolicy {
    static constexpr bool B_TRANSPOSE = true;
    static constexpr bool PARTIAL_TILES = true;
    static constexpr bool TRANSPOSED_STORE = false;
    static constexpr bool SHARE_B = false;
    static constexpr bool B_ROW_LIMIT = true; 
    struct Ctx : PolicyCtxBase {};
    static __device__ __forceinline__ Ctx make(const GemmParams& g, int which, int m0, int n0, int tid) {
        Ctx c;
        const int tn = n0 / GBN, b = tn / g.tiles_per_batch, c0 = (tn % g.tiles_per_batch) * GBN;
        c.rsA = make_rsrc(g.A[which], (unsigned)g.k * (unsigned)g.n * 2u);
        c.rsB = make_rsrc(g.B[which] + (long)b * g.n * g.dm, (unsigned)g.n * (unsigned)g.dm * 2u);
        c.voffA = ((m0 + (tid >> 3)) * g.n + 8 * (tid & 7)) * 2;
        c.a_qstride = 64 * g.n;
        // columns past dm (a ragged last tile) read the next position's values or zero: finite, and nobody
        // uses those columns of the result
        c.voffB = ((8 * (tid >> 5)) * g.dm + c0 + 8 * (tid & 31)) * 2;
        c.b_qstride = g.dm * 2;
        c.b_rows = g.n;
        return c;
    }
    static __device__ __forceinline__ int a_soff(const Ctx&, int step) { return step * (GBK * 2); }
    static __device__ __forceinline__ int b_soff(const Ctx& c, int step) { return step * GBK * c.b_qstride; }
};

// Paper-order path, second product: K' = Y W^K per head (Eq. 2: (E_1 K) W^K), all heads of a batch at
// once.  Rows = k projected slots of the three-term bf16 image of Y (row = [hi | mid | lo], 3*dm
// reduction slots, so that the products with the bf16 transform are exact in the fp32 accumulator),
// columns = (batch, head, t), B = the transform stored as (H*d, dm) rows (reduction contiguous), the
// reduction index wrapping around dm once per term.  Results leave as split partials in the projection's
// tile order, so the same finishing kernel takes over.
struct TransformPolicy {
    static constexpr bool B_TRANSPOSE = false;
    static constexpr bool PARTIAL_TILES = true;
    static constexpr bool TRANSPOSED_STORE = false;
    static constexpr bool SHARE_B = false;
    static constexpr bool B_ROW_LIMIT = false;
    struct Ctx : PolicyCtxBase { int steps_per_term; };
    static __device__ __forceinline__ Ctx make(const GemmParams& g, int which, int m0, int n0, int tid) {
        Ctx c;
        const int tn = n0 / GBN, b = tn / g.tiles_per_batch, c0 = (tn % g.tiles_per_batch) * GBN;
        const int row_bytes = 3 * g.dm * 2;
        c.rsA = make_rsrc(g.A[which] + (long)b * g.k * 3 * g.dm, (unsigned)g.k * (unsigned)row_bytes);
        c.rsB = make_rsrc(g.B[which], (unsigned)(g.tiles_per_batch * GBN) * (unsigned)g.dm * 2u);
        c.voffA = (m0 + (tid >> 3)) * row_bytes + 16 * (tid & 7);
        c.a_qstride = 32 * row_bytes;
        c.voffB = ((c0 + (tid >> 3)) * g.dm + 8 * (tid & 7)) * 2;
        c.b_qstride = 32 * g.dm * 2;
        c.steps_per_term = g.dm / GBK;
        return c;
    }
    static __device__ __forceinline__ int a_soff(const Ctx&, int step) { return step * (GBK * 2); }
    static __device__ __forceinline__ int b_soff(const Ctx& c, int step) { return (step % c.steps_per_term) * (GBK * 2); }
};

// dX = E^T dX': rows = (head, t) of the (BH*D x kp) image of (dX')^T, columns = sequence positions,
// reduction = projected slots (kp = k rounded up to 64, image zero-padded; rows of E past k read 0).
template <int D>
struct GradXPolicy {
    static constexpr bool B_TRANSPOSE = true;
    static constexpr bool PARTIAL_TILES = false;
    static constexpr bool TRANSPOSED_STORE = true;
    static constexpr bool SHARE_B = true;
    static constexpr bool B_ROW_LIMIT = false;
    struct Ctx : PolicyCtxBase {};
    static __device__ __forceinline__ Ctx make(const GemmParams& g, int which, int m0, int n0, int tid) {
        Ctx c;
        c.rsA = make_rsrc(g.A[which], (unsigned)(g.BH * D) * (unsigned)g.kp * 2u);
        c.rsB = make_rsrc(g.B[which], (unsigned)g.k * (unsigned)g.n * 2u);
        c.voffA = ((m0 + (tid >> 3)) * g.kp + 8 * (tid & 7)) * 2;
        c.a_qstride = 64 * g.kp;
        c.voffB = ((8 * (tid >> 5)) * g.n + n0 + 8 * (tid & 31)) * 2;
        c.b_qstride = g.n * 2;
        return c;
    }
    static __device__ __forceinline__ int a_soff(const Ctx&, int step) { return step * (GBK * 2); }
    static __device__ __forceinline__ int b_soff(const Ctx& c, int step) { return step * GBK * c.b_qstride; }
    // rows r0 + 8*k .. r0 + 8*k + 7 (64 rows from r0 lie inside one head) of column col, as 8 bf16
    static __device__ __forceinline__ void store_rows(const GemmParams& g, int which, int r0, int col, int k,
                                                      const uint4& v) {
        if (col >= g.n || r0 >= g.BH * D) return;
        const int bh = r0 / D, t = r0 % D + 8 * k;
        *(uint4*)((uint16_t*)g.C[which] + ((long)bh * g.n + col) * D + t) = v;
    }
};

// dE = sum_bh dX' X^T: rows = projected slots of the (BH, kp, D) image of dX', columns = sequence
// positions, reduction = (head, t) pairs, 64 of them per step.  FINAL: the reduction is not split, the
// bf16 result goes straight to dE / dF (k x n); otherwise fp32 split partials.
template <int D, bool FINAL = false>
struct GradEPolicy {
    static constexpr bool B_TRANSPOSE = false;
    static constexpr bool PARTIAL_TILES = !FINAL;
    static constexpr bool TRANSPOSED_STORE = false;
    static constexpr bool SHARE_B = true;
    static constexpr bool B_ROW_LIMIT = false;
    struct Ctx : PolicyCtxBase { int a_batch, b_batch; };
    static __device__ __forceinline__ Ctx make(const GemmParams& g, int which, int m0, int n0, int tid) {
        Ctx c;
        c.rsA = make_rsrc(g.A[which], (unsigned)g.BH * (unsigned)g.kp * (unsigned)(D * 2));
        c.rsB = make_rsrc(g.B[which], (unsigned)g.BH * (unsigned)g.n * (unsigned)(D * 2));
        c.voffA = ((m0 + (tid >> 3)) * D + 8 * (tid & 7)) * 2;
        c.a_qstride = 32 * D * 2;
        c.voffB = ((n0 + (tid >> 3)) * D + 8 * (tid & 7)) * 2;
        c.b_qstride = 32 * D * 2;
        c.a_batch = g.kp * D * 2;
        c.b_batch = g.n * D * 2;
        return c;
    }
    static __device__ __forceinline__ int a_soff(const Ctx& c, int step) {
        constexpr int spb = D / GBK;           // steps per head
        return (step / spb) * c.a_batch + (step % spb) * (GBK * 2);
    }
    static __device__ __forceinline__ int b_soff(const Ctx& c, int step) {
        constexpr int spb = D / GBK;
        return (step / spb) * c.b_batch + (step % spb) * (GBK * 2);
    }
    static __device__ __forceinline__ void store_groups(const GemmParams& g, const Ctx&, int which, int, int row,
                                                        int half, int col, const float (&ev)[4],
                                                        const float (&od)[4]) {
        // one 32-column segment of a row per half-wavefront and store
        if (col >= g.n) return;
        uint16_t* o = (uint16_t*)g.C[which] + col;
        const int r0 = row + 4 * half;
        const uint32_t pe[2] = {pack_bf16(ev[0], ev[1]), pack_bf16(ev[2], ev[3])};
        const uint32_t po[2] = {pack_bf16(od[0], od[1]), pack_bf16(od[2], od[3])};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (r0 + e < g.k) o[(long)(r0 + e) * g.n] = (uint16_t)(pe[e >> 1] >> (16 * (e & 1)));
            if (r0 + 8 + e < g.k) o[(long)(r0 + 8 + e) * g.n] = (uint16_t)(po[e >> 1] >> (16 * (e & 1)));
        }
    }
};

template <class Pol, bool STREAM>
static inline flurka_status launch_gemm_mfma_impl(const GemmParams& g, int grid, hipStream_t s) {
    auto kern = gemm_mfma_kernel<Pol, STREAM>;
    KernelFacts facts;
    if (!kernel_facts((const void*)kern, 256, G_LDS, &facts)) return FLURKA_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), G_LDS, s, g);
    if (hipGetLastError() != hipSuccess) return FLURKA_ERR_LAUNCH;
    return FLURKA_OK;
}

// One workgroup per item while the items fit one resident round; with more items than that (the short
// reductions of dK, dV), one resident round of workgroups that stream several items each.
template <class Pol>
static inline flurka_status launch_gemm_mfma(const GemmParams& g, hipStream_t s) {
    const long items = gemm_item_count<Pol>(g);
    int resident = resident_grid((const void*)gemm_mfma_kernel<Pol, true>, 256, G_LDS, items);
    if (resident < 1) return FLURKA_ERR_LAUNCH;
    // streaming needs a grid that is a multiple of 8: a workgroup's items then share id mod 8, and in
    // the SHARE_B order the ids past the last real item come last for every workgroup
    if (items > resident) resident = resident / 8 * 8;
    if (items <= resident || resident < 8) return launch_gemm_mfma_impl<Pol, false>(g, (int)items, s);
    return launch_gemm_mfma_impl<Pol, true>(g, resident, s);
}

// Split of one resident round of `resident` workgroups between two GEMMs of items_a items of steps_a
// reduction steps (items_a a multiple of 8) and items_b items of steps_b steps; `us` receives the time
// the model expects.  Measured on MI355X with operands from HBM: 1.8 us per reduction step of a
// workgroup that has a compute unit to itself, about 3 us for an epilogue that stores its accumulators
// as they are, 4.4 us for the transposing epilogue of dK, dV.
constexpr double G_STEP_US = 1.8, G_EPILOGUE_US = 3.0, G_EPILOGUE_T_US = 4.4;

inline PairPlan plan_pair(int items_a, int steps_a, int items_b, int steps_b, int resident, double* us) {
    const double ta = ((steps_a + 1) & ~1) * G_STEP_US + G_EPILOGUE_US;
    const double tb = ((steps_b + 1) & ~1) * G_STEP_US + G_EPILOGUE_T_US;
    PairPlan best{};
    double best_t = -1.0;
    for (int ba = 8; ba <= resident - 8; ba += 8) {
        if (ba > items_a && ba > 8) break;                      // more starters than first-part items
        const int bb = resident - ba;
        const double t_first = ((items_a + ba - 1) / ba) * ta;
        // items per workgroup of the second kind near the point where both kinds finish together
        const int x0 = (int)((t_first / tb * ba + items_b) / resident);
        for (int xb = x0 > 0 ? x0 : 1; xb <= x0 + 1; ++xb) {
            long main_b = (long)bb * xb / 8 * 8;
            if (main_b > items_b) main_b = items_b;
            const int xa = (int)((items_b - main_b + ba - 1) / ba);
            const double t_a = t_first + xa * tb, t_b = (double)((main_b + bb - 1) / bb) * tb;
            const double t = t_a > t_b ? t_a : t_b;
            if (best_t < 0.0 || t < best_t) {
                best_t = t;
                best.blocks_a = ba; best.main_b = (int)main_b; best.items_a = items_a; best.items_b = items_b;
            }
        }
    }
    if (us) *us = best_t;
    return best;
}

// Both GEMMs in one launch (gemm_mfma_pair_kernel) with the split `pl` of a resident round of
// `resident` workgroups (plan_pair).  Falls back to two launches where the kernel cannot keep 16
// workgroups resident.
template <class PolA, class PolB>
static inline flurka_status launch_gemm_mfma_pair(const GemmParams& ga, const GemmParams& gb, const PairPlan& pl,
                                                  int resident, hipStream_t s) {
    static_assert(PolA::SHARE_B && PolB::SHARE_B, "item counts and ranges in multiples of 8");
    auto kern = gemm_mfma_pair_kernel<PolA, PolB>;
    KernelFacts facts;
    if (!kernel_facts((const void*)kern, 256, G_LDS, &facts)) return FLURKA_ERR_LAUNCH;
    if ((long)facts.cus * facts.blocks_per_cu < resident || pl.blocks_a < 8 || pl.blocks_a > resident - 8) {
        const flurka_status st = launch_gemm_mfma<PolA>(ga, s);
        return st != FLURKA_OK ? st : launch_gemm_mfma<PolB>(gb, s);
    }
    int blocks_b = resident - pl.blocks_a;
    if (blocks_b > pl.main_b) blocks_b = pl.main_b > 0 ? pl.main_b : 0;
    hipLaunchKernelGGL(kern, dim3(pl.blocks_a + blocks_b), dim3(256), G_LDS, s, ga, gb, pl);
    if (hipGetLastError() != hipSuccess) return FLURKA_ERR_LAUNCH;
    return FLURKA_OK;
}

}  // namespace flurka
