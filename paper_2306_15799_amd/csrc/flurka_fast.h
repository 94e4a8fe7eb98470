// Declarations shared by the translation units of the bf16 MFMA path.
#pragma once

#include "flurka_mfma.h"

namespace flurka {

struct KeyStatePlan {
    int kpad;              // k rounded up to whole 32-key tiles
    int FT;                // 32-feature tiles
    int KR;                // key ranges handled by separate wavefronts and merged afterwards
    int tiles_per_range;
};
KeyStatePlan key_state_plan(const Problem& p);

// Device scratch of the key-state stage (all inside the caller's workspace).
struct KeyStateBuffers {
    uint16_t* Kimg;        // 3 x (BH, kpad, d) bf16
    uint32_t* Vimg;        // 2 x (BH, kpad/2, d) dwords
    float* nrm;            // (BH, kpad)
    float* Spart;          // (BH, KR, mf, d)
    float* zpart;          // (BH, KR, mf)
    float* cpart;          // (BH, KR, mf)
    uint16_t* St;          // (BH, d, mf) bf16, feature slots in operand order
    float* zp;             // (BH, mf)
    float* cp;             // (BH, mf)
};

// Sums the projection partials into ctx (K', V'), then fills S, z, c in ctx and the St/zp/cp images.
// `partials` points at split 0 of the [K' | V'] segments (ctx itself when splits == 1).
flurka_status fast_key_state(const Problem& p, const void* omega, float* ctx, const float* partials,
                             long split_stride, int splits, const KeyStateBuffers& b, hipStream_t s);

// Backward (flurka_bwd.hip)
bool fast_bwd_supported(const Problem& p);
size_t fast_bwd_ws_bytes(const Problem& p);

}  // namespace flurka
