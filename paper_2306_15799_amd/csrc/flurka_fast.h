// Declarations shared by the translation units of the bf16 MFMA path.
#pragma once

#include "flurka_mfma.h"

namespace flurka {

struct KeyStatePlan {
    int kpad;              // k rounded up to whole 32-key tiles
    int FT;                // 32-feature tiles
    int KR;                // key ranges = wavefronts of a workgroup, merged in LDS
    int tiles_per_range;
};
KeyStatePlan key_state_plan(const Problem& p);

// Device scratch of the key-state stage (all inside the caller's workspace).
struct KeyStateBuffers {
    uint16_t* Kimg;        // 3 x (BH, kpad * d) bf16, key_state's operand order (see proj_finish_kernel)
    uint32_t* Vimg;        // 2 x (BH, kpad/2, d) dwords
    float* nrm;            // (BH, kpad)
    uint16_t* St;          // (BH, d, mf) bf16, feature slots in operand order; performer: S_j / z_j
    float* zp;             // (BH, mf)
    uint16_t* cw;          // (BH, mf, 4) bf16: hi, mid, lo terms of c + ln z, then 0 (performer only)
};

// Sums the projection's tile-ordered split partials (tilesM x tilesN tiles per split and tensor) into
// ctx (K', V'), then fills S, z, c in ctx and the St/zp/cw images.
flurka_status fast_key_state(const Problem& p, const void* omega, float* ctx, const float* partials,
                             int tilesM, int tilesN, int splits, const KeyStateBuffers& b, hipStream_t s);

// Kernel attention without a sequence projection (p.k == p.n, K' = K, V' = V): packs the caller's bf16
// K, V into the key-state operand images and fills S, z, c in ctx and the St/zp/cw images.
flurka_status fast_identity_key_state(const Problem& p, const void* K, const void* V, const void* omega, float* S,
                                      float* z, float* c, const KeyStateBuffers& b, hipStream_t s);
// The projection's second stage alone: sums the split partials into K', V' (ctx) and, with `images`,
// writes the key-state operand images.
flurka_status fast_proj_finish(const Problem& p, float* ctx, const float* partials, int tilesM, int tilesN,
                               int splits, bool images, const KeyStateBuffers& b, hipStream_t s);

// Grid of a kernel whose workgroups split `items` evenly among themselves: as many workgroups as the
// device keeps resident at once for this block size and LDS use (one round, no tail), at most `items`.
// Returns 0 if the runtime cannot place the kernel.
inline int resident_grid(const void* kernel, int threads, int lds_bytes, long items) {
    KernelFacts f;
    if (!kernel_facts(kernel, threads, lds_bytes, &f)) return 0;
    long grid = (long)f.cus * f.blocks_per_cu;
    if (grid > items) grid = items;
    return (int)grid;
}

// Backward (flurka_bwd.hip)
bool fast_bwd_supported(const Problem& p);
size_t fast_bwd_ws_bytes(const Problem& p);

}  // namespace flurka
