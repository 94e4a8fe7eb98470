// Internal declarations shared by the translation units of libflurka.
// Nothing here is part of the public ABI (that is include/flurka.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "flurka.h"

namespace flurka {

// Problem description after validation.
struct Problem {
    int B, H, n, d, k, m;
    int mf;              // feature count: m (performer) or d (elu1)
    int mfp;             // mf rounded up to whole 32-feature tiles (image strides of the MFMA forward)
    int BH;
    int omega_per_head;
    int bf16;            // storage type of caller tensors
    int elu;             // feature map
    // options of the extended entry points (generic kernels only)
    int ef_per_head;     // E, F (and dE, dF) are (H, k, n): one pair per head
    int grad_ef_f32;     // dE, dF are written as float32 whatever the storage type
};

static inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Context buffer (float32): state carried from forward to backward.
// Every segment starts on a 256-byte boundary.
struct CtxLayout {
    size_t Kp, Vp, S, z, c, lse, total;   // offsets / total in floats
};

static inline CtxLayout ctx_layout(const Problem& p) {
    CtxLayout L;
    size_t o = 0;
    const size_t BH = (size_t)p.BH;
    L.Kp = o;   o += round_up(BH * p.k * p.d, 64);
    L.Vp = o;   o += round_up(BH * p.k * p.d, 64);
    L.S = o;    o += round_up(BH * p.mf * p.d, 64);
    L.z = o;    o += round_up(BH * p.mf, 64);
    L.c = o;    o += round_up(BH * p.mf, 64);   // exponent shift per (batch, head, feature)
    L.lse = o;  o += round_up(BH * p.n, 64);    // log of the denominator per query row
    L.total = o;
    return L;
}

// ---- generic (fp32-arithmetic) path ---------------------------------------
// Rows of Q handled per chunk so that the (B,H,rows,mf) feature buffer stays
// near 128 MiB whatever n is.
static inline int generic_chunk_rows(const Problem& p) {
    const size_t budget = (size_t)128 << 20;
    size_t rows = budget / (4 * (size_t)p.BH * (size_t)p.mf);
    if (rows < 64) rows = 64;
    rows = rows / 64 * 64;
    if (rows > (size_t)p.n) rows = (size_t)p.n;
    return (int)rows;
}

struct GenericWs {
    size_t P, T, N, PhiK, dD, dS, dz, dPhiK, dKp, dVp, rs, total;   // floats
};

static inline GenericWs generic_ws_layout(const Problem& p, int bwd) {
    GenericWs W{};
    const size_t BH = (size_t)p.BH;
    const size_t nc = (size_t)generic_chunk_rows(p);
    size_t o = 0;
    W.P = o; o += round_up(BH * nc * p.mf, 64);
    W.N = o; o += round_up(BH * nc * p.d, 64);
    W.PhiK = o; o += round_up(BH * p.k * p.mf, 64);
    if (bwd) {
        W.T = o;     o += round_up(BH * nc * p.mf, 64);
        W.dD = o;    o += round_up(BH * nc, 64);
        W.dS = o;    o += round_up(BH * p.mf * p.d, 64);
        W.dz = o;    o += round_up(BH * p.mf, 64);
        W.dPhiK = o; o += round_up(BH * p.k * p.mf, 64);
        W.dKp = o;   o += round_up(BH * p.k * p.d, 64);
        W.dVp = o;   o += round_up(BH * p.k * p.d, 64);
        W.rs = o;    o += round_up(BH * p.k, 64);
    }
    W.total = o;
    return W;
}

struct FwdArgs {
    const void *Q, *K, *V, *E, *F, *omega;
    void* out;
    float* ctx;
    float* ws;
};

struct BwdArgs {
    const void *Q, *K, *V, *E, *F, *omega, *out, *dOut;
    const float* ctx;
    void *dQ, *dK, *dV, *dE, *dF;
    float* ws;
    float* dOmega;       // optional (extended entry point): d loss / d omega, (H|1, m, d) float32
};

// Each returns FLURKA_OK or FLURKA_ERR_LAUNCH.
flurka_status generic_forward(const Problem& p, const FwdArgs& a, hipStream_t s);
flurka_status generic_backward(const Problem& p, const BwdArgs& a, hipStream_t s);
flurka_status generic_backward_from(const Problem& p, const BwdArgs& a, hipStream_t s, int query_done);

// ---- stage timer -------------------------------------------------------------
enum Stage {
    STAGE_PROJECT = 0,     // K' = E K and V' = F V
    STAGE_KEY_STATE = 1,   // PhiK, S, z
    STAGE_QUERY = 2,       // phi(Q), numerator, denominator, out
    STAGE_BWD_QUERY = 3,   // recompute P; dQ, dS, dz
    STAGE_BWD_KEY = 4,     // dPhiK, dV', dK'
    STAGE_BWD_DKDV = 5,    // dK = E^T dK', dV = F^T dV'
    STAGE_BWD_DEDF = 6,    // dE, dF
    // single kernels of the MFMA path (reported as "stage:kernel")
    STAGE_K_PROJ_GEMM = 7,
    STAGE_K_PROJ_FINISH = 8,
    STAGE_K_KEY_STATE = 9,
    STAGE_K_MERGE_PACK = 10,
    STAGE_K_QUERY_STREAM = 11,
    STAGE_K_BWD_X = 13,
    STAGE_K_BWD_Y = 14,
    STAGE_K_BWD_MERGE = 15,
    STAGE_K_BWD_KEY = 16,
    STAGE_K_GRAD_X = 17,
    STAGE_K_GRAD_E = 18,
    STAGE_K_SUM_SPLITS = 19,
    STAGE_BWD_GRADS = 20,  // dK, dV, dE, dF together (MFMA path: one launch)
    STAGE_K_GRAD_PAIR = 21,
    STAGE_K_WIDE_GEMM = 22,        // paper-order path: Y = E X on the model-wide input
    STAGE_K_WIDE_FINISH = 23,
    STAGE_K_TRANSFORM_GEMM = 24,   // K' = Y W^K, V' = Y W^V
    STAGE_K_IDENTITY_PACK = 25,    // baselines: operand images of K, V without a projection
    STAGE_K_LINFORMER_PACK = 26,   // baselines: K', V' as the query stream's images
    STAGE_COUNT = 27
};
// No-ops unless the timer is enabled.  begin/end pairs must not nest.
void stage_begin(hipStream_t s);
void stage_end(hipStream_t s, Stage id);
// Forgets a begin that never saw its end (a call that returned early on a launch error).
void stage_abandon();

struct StageScope {
    hipStream_t s; Stage id;
    StageScope(hipStream_t s_, Stage id_) : s(s_), id(id_) { stage_begin(s); }
    ~StageScope() { stage_end(s, id); }
};

// ---- launch facts ------------------------------------------------------------
// What the runtime reports about a kernel for one (device, block size, dynamic LDS size) does not
// change while the process lives, so it is asked once and kept in a host-side table (no device memory).
struct KernelFacts {
    int cus;             // compute units of the device
    int blocks_per_cu;   // workgroups of this kernel a compute unit holds at once
};
// First use on the current device raises the kernel's dynamic-LDS limit to `lds_bytes` and queries its
// occupancy; every later call is a table lookup.  false: the runtime refused.
bool kernel_facts(const void* kernel, int threads, int lds_bytes, KernelFacts* out);
// Compute units of the current device; 256 (MI355X) where no device is visible, so that buffer sizes
// can still be computed on a host without a GPU.
int chip_cus();

// ---- bf16 MFMA path ---------------------------------------------------------
// Whether the MFMA kernels cover the problem (dtype, feature map, tile multiples).
bool fast_supported(const Problem& p, int bwd);
// 16-byte alignment of the caller tensors the vector loads touch (nullptr entries are skipped).
bool fast_pointers_ok(const void* a, const void* b, const void* c, const void* d, const void* e,
                      const void* f, const void* g);
size_t fast_ws_bytes(const Problem& p, int bwd);
flurka_status fast_forward(const Problem& p, const FwdArgs& a, hipStream_t s);
flurka_status fast_backward(const Problem& p, const BwdArgs& a, hipStream_t s);
// Paper-order forward: K' = (E X_K) W^K, V' = (F X_V) W^V from the model-wide inputs.
struct FusedWArgs {
    const void *Q, *XK, *XV, *E, *F, *WK, *WV, *omega;
    void* out;
    float* ctx;
    float* ws;
    int dm;
};
bool fast_fusedw_supported(const Problem& p, int dm);
size_t fast_fusedw_ws_bytes(const Problem& p, int dm);
flurka_status fast_forward_fusedw(const Problem& p, const FusedWArgs& a, hipStream_t s);
// Comparison baselines (flurka_baseline_* entry points); `which` is a flurka_baseline value.
bool fast_baseline_supported(int which, const Problem& p);
size_t fast_baseline_ws_bytes(int which, const Problem& p);
size_t fast_baseline_ctx_floats(int which, const Problem& p);
flurka_status fast_kernel_attn_forward(const Problem& p, const FwdArgs& a, hipStream_t s);   // p.k == p.n
flurka_status fast_linformer_forward(const Problem& p, const FwdArgs& a, hipStream_t s);
// Key-side state from K', V' already in ctx: PhiK (scratch, BH*k*mf floats), S, z and the shifts c.
flurka_status generic_key_state(const Problem& p, const void* omega, float* ctx, float* PhiK, hipStream_t s);

// ---- device helpers --------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(((uint32_t)b) << 16);
}

// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float load_elem(const void* p, long i, int bf16) {
    return bf16 ? bf16_to_f32(((const uint16_t*)p)[i]) : ((const float*)p)[i];
}

__device__ __forceinline__ void store_elem(void* p, long i, float v, int bf16) {
    if (bf16) ((uint16_t*)p)[i] = f32_to_bf16(v);
    else ((float*)p)[i] = v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace flurka
