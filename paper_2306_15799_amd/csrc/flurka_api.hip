// C ABI of libflurka: argument validation, buffer sizing and dispatch.
// The entry points are documented in include/flurka.h.
#include "flurka_internal.h"

#include <mutex>
#include <vector>

using namespace flurka;

// ---- stage timer ---------------------------------------------------------------
namespace flurka {
namespace {
constexpr int kMaxIntervals = 4096;
bool g_prof_on = false;
std::vector<hipEvent_t> g_events;       // 2 * kMaxIntervals, created on enable
std::vector<int> g_stage_of;            // stage id per recorded interval
int g_intervals = 0;
bool g_open = false;
}  // namespace

void stage_begin(hipStream_t s) {
    if (!g_prof_on || g_intervals >= kMaxIntervals) return;
    if (hipEventRecord(g_events[2 * g_intervals], s) == hipSuccess) g_open = true;
}

void stage_end(hipStream_t s, Stage id) {
    if (!g_prof_on || !g_open) return;
    g_open = false;
    if (hipEventRecord(g_events[2 * g_intervals + 1], s) != hipSuccess) return;
    g_stage_of[g_intervals] = (int)id;
    ++g_intervals;
}

void stage_abandon() { g_open = false; }

// ---- launch facts ---------------------------------------------------------------
namespace {
struct FactsEntry { int dev; const void* kernel; int threads, lds; KernelFacts facts; };
std::mutex g_facts_mutex;
std::vector<FactsEntry> g_facts;         // a few dozen entries at most: linear search
std::vector<int> g_cus;                  // compute units per device id, 0 = not asked yet

// compute units of device `dev`; 0 if the runtime cannot tell (g_facts_mutex held)
int cus_of(int dev) {
    if (dev < 0) return 0;
    if ((size_t)dev >= g_cus.size()) g_cus.resize((size_t)dev + 1, 0);
    if (g_cus[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return 0;
        g_cus[dev] = cus;
    }
    return g_cus[dev];
}
}  // namespace

bool kernel_facts(const void* kernel, int threads, int lds_bytes, KernelFacts* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(g_facts_mutex);
    for (const FactsEntry& e : g_facts)
        if (e.dev == dev && e.kernel == kernel && e.threads == threads && e.lds == lds_bytes) {
            *out = e.facts;
            return true;
        }
    KernelFacts f{};
    f.cus = cus_of(dev);
    if (f.cus < 1) return false;
    if (lds_bytes > 0 &&
        hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes) != hipSuccess)
        return false;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&f.blocks_per_cu, kernel, threads, (size_t)lds_bytes) != hipSuccess ||
        f.blocks_per_cu < 1)
        return false;
    g_facts.push_back(FactsEntry{dev, kernel, threads, lds_bytes, f});
    *out = f;
    return true;
}

int chip_cus() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return 256; }
    std::lock_guard<std::mutex> lock(g_facts_mutex);
    const int cus = cus_of(dev);
    if (cus < 1) { (void)hipGetLastError(); return 256; }
    return cus;
}
}  // namespace flurka

namespace {

constexpr int kVersion = 150;

flurka_status make_problem(int B, int H, int n, int d, int k, int m, int omega_per_head,
                           int dtype, int phi, Problem* out) {
    if (dtype != FLURKA_F32 && dtype != FLURKA_BF16) return FLURKA_ERR_DTYPE;
    if (phi != FLURKA_PHI_PERFORMER && phi != FLURKA_PHI_ELU1) return FLURKA_ERR_DTYPE;
    if (B < 1 || H < 1 || n < 1 || d < 1 || k < 1 || m < 1) return FLURKA_ERR_SHAPE;
    if ((long)B * (long)H > FLURKA_MAX_BATCH_HEADS) return FLURKA_ERR_SHAPE;
    if (d > FLURKA_MAX_FEATURE_DIM || m > FLURKA_MAX_FEATURE_DIM) return FLURKA_ERR_SHAPE;
    if (n > FLURKA_MAX_SEQ || k > FLURKA_MAX_SEQ) return FLURKA_ERR_SHAPE;
    if (phi == FLURKA_PHI_ELU1 && m != d) return FLURKA_ERR_SHAPE;
    Problem p;
    p.B = B; p.H = H; p.n = n; p.d = d; p.k = k; p.m = m;
    p.elu = (phi == FLURKA_PHI_ELU1);
    p.mf = p.elu ? d : m;
    p.mfp = (p.mf + 31) / 32 * 32;
    p.BH = B * H;
    p.omega_per_head = omega_per_head ? 1 : 0;
    p.bf16 = (dtype == FLURKA_BF16);
    p.ef_per_head = 0;
    p.grad_ef_f32 = 0;
    *out = p;
    return FLURKA_OK;
}

bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

bool valid_algo(int a) { return a == FLURKA_ALGO_AUTO || a == FLURKA_ALGO_GENERIC || a == FLURKA_ALGO_FAST; }

}  // namespace

// Scratch of flurka_attn_fwd_static: part of the library's device image, so every GPU the library runs
// on holds its own copy at its own address until the process ends.  In host code the array's name only
// stands for the symbol; its device address is asked from the runtime once per device and kept.
static __device__ __align__(256) unsigned char scratch[FLURKA_STATIC_WORKSPACE_BYTES];

namespace {
std::mutex g_scratch_mutex;
std::vector<void*> g_scratch_ptr;        // per device id, nullptr = not asked yet

// device address of `scratch` on the current device, or nullptr if the runtime cannot tell
void* static_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if ((size_t)dev >= g_scratch_ptr.size()) g_scratch_ptr.resize((size_t)dev + 1, nullptr);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// Validation and dispatch shared by the two forward entry points.  `workspace == nullptr` stands for
// the library's own scratch array (looked up only after everything else has been validated).
flurka_status forward_impl(const void* Q, const void* K, const void* V, const void* E, const void* F,
                           const void* omega, void* out, void* ctx, size_t ctx_bytes, void* workspace,
                           size_t workspace_bytes, bool own_scratch, int B, int H, int n, int d, int k, int m,
                           int omega_per_head, flurka_dtype dtype, flurka_phi phi, flurka_algo algo, void* stream,
                           const flurka_options* opt = nullptr) {
    Problem p;
    flurka_status st = make_problem(B, H, n, d, k, m, omega_per_head, dtype, phi, &p);
    if (st != FLURKA_OK) return st;
    if (!valid_algo(algo)) return FLURKA_ERR_DTYPE;
    if (opt) p.ef_per_head = opt->ef_per_head ? 1 : 0;      // the other options concern the backward only
    if (!Q || !K || !V || !E || !F || !out || !ctx || (!own_scratch && !workspace)) return FLURKA_ERR_NULL;
    if (!p.elu && !omega) return FLURKA_ERR_NULL;
    const size_t es = p.bf16 ? 2 : 4;
    if (misaligned(Q, es) || misaligned(K, es) || misaligned(V, es) || misaligned(E, es) ||
        misaligned(F, es) || misaligned(out, es) || (omega && misaligned(omega, es)) ||
        misaligned(ctx, 256) || (!own_scratch && misaligned(workspace, 256)))
        return FLURKA_ERR_ALIGN;
    const bool fast_ok = !p.ef_per_head && fast_supported(p, 0) && fast_pointers_ok(Q, K, V, E, F, omega, out);
    if (algo == FLURKA_ALGO_FAST && !fast_ok) return FLURKA_ERR_UNSUPPORTED;
    const bool use_fast = (algo != FLURKA_ALGO_GENERIC) && fast_ok;
    if (ctx_bytes < ctx_layout(p).total * sizeof(float)) return FLURKA_ERR_WORKSPACE;
    const size_t need = use_fast ? fast_ws_bytes(p, 0) : generic_ws_layout(p, 0).total * sizeof(float);
    if (workspace_bytes < need) return FLURKA_ERR_WORKSPACE;
    if (own_scratch && !(workspace = static_scratch())) return FLURKA_ERR_LAUNCH;

    FwdArgs a{Q, K, V, E, F, omega, out, (float*)ctx, (float*)workspace};
    hipStream_t s = (hipStream_t)stream;
    st = use_fast ? fast_forward(p, a, s) : generic_forward(p, a, s);
    if (st != FLURKA_OK) stage_abandon();
    return st;
}
}  // namespace

extern "C" {

int flurka_version(void) { return kVersion; }

const char* flurka_status_str(flurka_status s) {
    switch (s) {
        case FLURKA_OK: return "ok";
        case FLURKA_ERR_NULL: return "required pointer is NULL";
        case FLURKA_ERR_SHAPE: return "invalid shape";
        case FLURKA_ERR_DTYPE: return "unknown dtype, feature map or algo";
        case FLURKA_ERR_UNSUPPORTED: return "problem not supported by the selected algo";
        case FLURKA_ERR_WORKSPACE: return "ctx or workspace buffer too small";
        case FLURKA_ERR_LAUNCH: return "HIP launch error";
        case FLURKA_ERR_ALIGN: return "misaligned pointer";
    }
    return "unknown status";
}

size_t flurka_ctx_bytes(int B, int H, int n, int d, int k, int m, flurka_dtype dtype, flurka_phi phi) {
    Problem p;
    if (make_problem(B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    return ctx_layout(p).total * sizeof(float);
}

flurka_status flurka_ctx_layout(int B, int H, int n, int d, int k, int m, flurka_dtype dtype,
                                flurka_phi phi, size_t* offsets6) {
    if (!offsets6) return FLURKA_ERR_NULL;
    Problem p;
    flurka_status st = make_problem(B, H, n, d, k, m, 1, dtype, phi, &p);
    if (st != FLURKA_OK) return st;
    const CtxLayout L = ctx_layout(p);
    offsets6[0] = L.Kp; offsets6[1] = L.Vp; offsets6[2] = L.S; offsets6[3] = L.z; offsets6[4] = L.c;
    offsets6[5] = L.lse;
    return FLURKA_OK;
}

int flurka_fast_path_supported(int B, int H, int n, int d, int k, int m, flurka_dtype dtype,
                               flurka_phi phi, flurka_pass pass) {
    Problem p;
    if (make_problem(B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    if (pass != FLURKA_PASS_FWD && pass != FLURKA_PASS_BWD) return 0;
    return fast_supported(p, pass == FLURKA_PASS_BWD) ? 1 : 0;
}

size_t flurka_workspace_bytes(int B, int H, int n, int d, int k, int m, flurka_dtype dtype,
                              flurka_phi phi, flurka_pass pass, flurka_algo algo) {
    Problem p;
    if (make_problem(B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    if (pass != FLURKA_PASS_FWD && pass != FLURKA_PASS_BWD) return 0;
    if (!valid_algo(algo)) return 0;
    const int bwd = (pass == FLURKA_PASS_BWD);
    const size_t gen = generic_ws_layout(p, bwd).total * sizeof(float);
    const size_t fast = fast_supported(p, bwd) ? fast_ws_bytes(p, bwd) : 0;
    if (algo == FLURKA_ALGO_GENERIC) return gen;
    if (algo == FLURKA_ALGO_FAST) return fast;
    return fast > gen ? fast : gen;
}

flurka_status flurka_attn_fwd(const void* Q, const void* K, const void* V, const void* E, const void* F,
                              const void* omega, void* out, void* ctx, size_t ctx_bytes, void* workspace,
                              size_t workspace_bytes, int B, int H, int n, int d, int k, int m,
                              int omega_per_head, flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                              void* stream) {
    return forward_impl(Q, K, V, E, F, omega, out, ctx, ctx_bytes, workspace, workspace_bytes, false, B, H, n, d,
                        k, m, omega_per_head, dtype, phi, algo, stream);
}

flurka_status flurka_attn_fwd_static(const void* Q, const void* K, const void* V, const void* E, const void* F,
                                     const void* omega, void* out, void* ctx, size_t ctx_bytes, int B, int H,
                                     int n, int d, int k, int m, int omega_per_head, flurka_dtype dtype,
                                     flurka_phi phi, flurka_algo algo, void* stream) {
    return forward_impl(Q, K, V, E, F, omega, out, ctx, ctx_bytes, nullptr, FLURKA_STATIC_WORKSPACE_BYTES, true, B,
                        H, n, d, k, m, omega_per_head, dtype, phi, algo, stream);
}

int flurka_fused_w_supported(int B, int H, int n, int d, int k, int m, int dm, flurka_dtype dtype, flurka_phi phi) {
    Problem p;
    if (make_problem(B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    if (dm < 1 || dm > (1 << 20)) return 0;
    return fast_fusedw_supported(p, dm) ? 1 : 0;
}

size_t flurka_fused_w_workspace_bytes(int B, int H, int n, int d, int k, int m, int dm, flurka_dtype dtype,
                                      flurka_phi phi) {
    Problem p;
    if (make_problem(B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    if (dm < 1 || dm > (1 << 20) || !fast_fusedw_supported(p, dm)) return 0;
    return fast_fusedw_ws_bytes(p, dm);
}

flurka_status flurka_attn_fwd_fused_w(const void* Q, const void* XK, const void* XV, const void* E, const void* F,
                                      const void* WK, const void* WV, const void* omega, void* out, void* ctx,
                                      size_t ctx_bytes, void* workspace, size_t workspace_bytes, int B, int H, int n,
                                      int d, int k, int m, int dm, int omega_per_head, flurka_dtype dtype,
                                      flurka_phi phi, void* stream) {
    Problem p;
    flurka_status st = make_problem(B, H, n, d, k, m, omega_per_head, dtype, phi, &p);
    if (st != FLURKA_OK) return st;
    if (dm < 1 || dm > (1 << 20)) return FLURKA_ERR_SHAPE;
    if (!Q || !XK || !XV || !E || !F || !WK || !WV || !out || !ctx || !workspace) return FLURKA_ERR_NULL;
    if (!p.elu && !omega) return FLURKA_ERR_NULL;
    if (misaligned(ctx, 256) || misaligned(workspace, 256)) return FLURKA_ERR_ALIGN;
    const size_t es = p.bf16 ? 2 : 4;
    if (misaligned(Q, es) || misaligned(XK, es) || misaligned(XV, es) || misaligned(E, es) || misaligned(F, es) ||
        misaligned(WK, es) || misaligned(WV, es) || misaligned(out, es) || (omega && misaligned(omega, es)))
        return FLURKA_ERR_ALIGN;
    if (!fast_fusedw_supported(p, dm) || !fast_pointers_ok(Q, XK, XV, E, F, omega, out) ||
        !fast_pointers_ok(WK, WV, nullptr, nullptr, nullptr, nullptr, nullptr))
        return FLURKA_ERR_UNSUPPORTED;
    if (ctx_bytes < ctx_layout(p).total * sizeof(float)) return FLURKA_ERR_WORKSPACE;
    if (workspace_bytes < fast_fusedw_ws_bytes(p, dm)) return FLURKA_ERR_WORKSPACE;
    FusedWArgs a{Q, XK, XV, E, F, WK, WV, omega, out, (float*)ctx, (float*)workspace, dm};
    st = fast_forward_fusedw(p, a, (hipStream_t)stream);
    if (st != FLURKA_OK) stage_abandon();
    return st;
}

namespace {
// Problem of a baseline call: kernel attention has every position as a key; Linformer has one "feature"
// per key and no feature map of its own.
flurka_status baseline_problem(int which, int B, int H, int n, int d, int k, int m, int omega_per_head, int dtype,
                               int phi, Problem* p) {
    if (which == FLURKA_BASELINE_KERNEL_ATTN) return make_problem(B, H, n, d, n, m, omega_per_head, dtype, phi, p);
    if (which == FLURKA_BASELINE_LINFORMER) return make_problem(B, H, n, d, k, 32, 1, dtype, FLURKA_PHI_PERFORMER, p);
    return FLURKA_ERR_DTYPE;
}
}  // namespace

int flurka_baseline_supported(flurka_baseline which, int B, int H, int n, int d, int k, int m, flurka_dtype dtype,
                              flurka_phi phi) {
    Problem p;
    if (baseline_problem(which, B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    return fast_baseline_supported(which, p) ? 1 : 0;
}

size_t flurka_baseline_ctx_bytes(flurka_baseline which, int B, int H, int n, int d, int k, int m, flurka_dtype dtype,
                                 flurka_phi phi) {
    Problem p;
    if (baseline_problem(which, B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    return fast_baseline_ctx_floats(which, p) * sizeof(float);
}

size_t flurka_baseline_workspace_bytes(flurka_baseline which, int B, int H, int n, int d, int k, int m,
                                       flurka_dtype dtype, flurka_phi phi) {
    Problem p;
    if (baseline_problem(which, B, H, n, d, k, m, 1, dtype, phi, &p) != FLURKA_OK) return 0;
    if (!fast_baseline_supported(which, p)) return 0;
    return fast_baseline_ws_bytes(which, p);
}

flurka_status flurka_baseline_fwd(flurka_baseline which, const void* Q, const void* K, const void* V, const void* E,
                                  const void* F, const void* omega, void* out, void* ctx, size_t ctx_bytes,
                                  void* workspace, size_t workspace_bytes, int B, int H, int n, int d, int k, int m,
                                  int omega_per_head, flurka_dtype dtype, flurka_phi phi, void* stream) {
    Problem p;
    flurka_status st = baseline_problem(which, B, H, n, d, k, m, omega_per_head, dtype, phi, &p);
    if (st != FLURKA_OK) return st;
    const bool lin = which == FLURKA_BASELINE_LINFORMER;
    if (!Q || !K || !V || !out || !ctx || !workspace) return FLURKA_ERR_NULL;
    if (lin && (!E || !F)) return FLURKA_ERR_NULL;
    if (!lin && !p.elu && !omega) return FLURKA_ERR_NULL;
    if (misaligned(ctx, 256) || misaligned(workspace, 256)) return FLURKA_ERR_ALIGN;
    if (!fast_baseline_supported(which, p) ||
        !fast_pointers_ok(Q, K, V, lin ? E : nullptr, lin ? F : nullptr, lin ? nullptr : omega, out))
        return FLURKA_ERR_UNSUPPORTED;
    if (ctx_bytes < fast_baseline_ctx_floats(which, p) * sizeof(float)) return FLURKA_ERR_WORKSPACE;
    if (workspace_bytes < fast_baseline_ws_bytes(which, p)) return FLURKA_ERR_WORKSPACE;
    FwdArgs a{Q, K, V, E, F, omega, out, (float*)ctx, (float*)workspace};
    st = lin ? fast_linformer_forward(p, a, (hipStream_t)stream) : fast_kernel_attn_forward(p, a, (hipStream_t)stream);
    if (st != FLURKA_OK) stage_abandon();
    return st;
}

namespace {
flurka_status backward_impl(const void* Q, const void* K, const void* V, const void* E, const void* F,
                            const void* omega, const void* out, const void* dOut, const void* ctx,
                            size_t ctx_bytes, void* dQ, void* dK, void* dV, void* dE, void* dF, void* workspace,
                            size_t workspace_bytes, int B, int H, int n, int d, int k, int m, int omega_per_head,
                            flurka_dtype dtype, flurka_phi phi, flurka_algo algo, void* stream,
                            const flurka_options* opt) {
    Problem p;
    flurka_status st = make_problem(B, H, n, d, k, m, omega_per_head, dtype, phi, &p);
    if (st != FLURKA_OK) return st;
    if (!valid_algo(algo)) return FLURKA_ERR_DTYPE;
    void* d_omega = nullptr;
    if (opt) {
        p.ef_per_head = opt->ef_per_head ? 1 : 0;
        p.grad_ef_f32 = opt->grad_ef_f32 ? 1 : 0;
        d_omega = opt->d_omega;
    }
    if (!Q || !K || !V || !E || !F || !out || !dOut || !ctx || !dQ || !dK || !dV || !dE || !dF || !workspace)
        return FLURKA_ERR_NULL;
    if (!p.elu && !omega) return FLURKA_ERR_NULL;
    if (d_omega && p.elu) return FLURKA_ERR_SHAPE;            // the elu1 map has no omega
    const size_t es = p.bf16 ? 2 : 4;
    const size_t ges = p.grad_ef_f32 ? 4 : es;
    if (misaligned(Q, es) || misaligned(K, es) || misaligned(V, es) || misaligned(E, es) ||
        misaligned(F, es) || misaligned(out, es) || misaligned(dOut, es) || (omega && misaligned(omega, es)) ||
        misaligned(dQ, es) || misaligned(dK, es) || misaligned(dV, es) || misaligned(dE, ges) ||
        misaligned(dF, ges) || misaligned(d_omega, 4) || misaligned(ctx, 256) || misaligned(workspace, 256))
        return FLURKA_ERR_ALIGN;
    const bool plain = !p.ef_per_head && !p.grad_ef_f32 && !d_omega;      // the options run on the generic kernels
    const bool fast_ok = plain && fast_supported(p, 1) && fast_pointers_ok(Q, K, V, E, F, omega, dOut) &&
                         fast_pointers_ok(dQ, dK, dV, dE, dF, nullptr, out);
    if (algo == FLURKA_ALGO_FAST && !fast_ok) return FLURKA_ERR_UNSUPPORTED;
    const bool use_fast = (algo != FLURKA_ALGO_GENERIC) && fast_ok;
    if (ctx_bytes < ctx_layout(p).total * sizeof(float)) return FLURKA_ERR_WORKSPACE;
    const size_t need = use_fast ? fast_ws_bytes(p, 1) : generic_ws_layout(p, 1).total * sizeof(float);
    if (workspace_bytes < need) return FLURKA_ERR_WORKSPACE;

    BwdArgs a{Q, K, V, E, F, omega, out, dOut, (const float*)ctx, dQ, dK, dV, dE, dF, (float*)workspace, (float*)d_omega};
    hipStream_t s = (hipStream_t)stream;
    st = use_fast ? fast_backward(p, a, s) : generic_backward(p, a, s);
    if (st != FLURKA_OK) stage_abandon();
    return st;
}
}  // namespace

flurka_status flurka_attn_bwd(const void* Q, const void* K, const void* V, const void* E, const void* F,
                              const void* omega, const void* out, const void* dOut, const void* ctx,
                              size_t ctx_bytes, void* dQ, void* dK, void* dV, void* dE, void* dF, void* workspace,
                              size_t workspace_bytes, int B, int H, int n, int d, int k, int m,
                              int omega_per_head, flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                              void* stream) {
    return backward_impl(Q, K, V, E, F, omega, out, dOut, ctx, ctx_bytes, dQ, dK, dV, dE, dF, workspace, workspace_bytes,
                         B, H, n, d, k, m, omega_per_head, dtype, phi, algo, stream, nullptr);
}

flurka_status flurka_attn_fwd_ex(const void* Q, const void* K, const void* V, const void* E, const void* F,
                                 const void* omega, void* out, void* ctx, size_t ctx_bytes, void* workspace,
                                 size_t workspace_bytes, int B, int H, int n, int d, int k, int m,
                                 int omega_per_head, flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                                 const flurka_options* options, void* stream) {
    return forward_impl(Q, K, V, E, F, omega, out, ctx, ctx_bytes, workspace, workspace_bytes, false, B, H, n, d,
                        k, m, omega_per_head, dtype, phi, algo, stream, options);
}

flurka_status flurka_attn_bwd_ex(const void* Q, const void* K, const void* V, const void* E, const void* F,
                                 const void* omega, const void* out, const void* dOut, const void* ctx,
                                 size_t ctx_bytes, void* dQ, void* dK, void* dV, void* dE, void* dF, void* workspace,
                                 size_t workspace_bytes, int B, int H, int n, int d, int k, int m,
                                 int omega_per_head, flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                                 const flurka_options* options, void* stream) {
    return backward_impl(Q, K, V, E, F, omega, out, dOut, ctx, ctx_bytes, dQ, dK, dV, dE, dF, workspace, workspace_bytes,
                         B, H, n, d, k, m, omega_per_head, dtype, phi, algo, stream, options);
}

flurka_status flurka_profile_enable(int on) {
    if (on && !g_prof_on) {
        g_events.resize(2 * kMaxIntervals);
        g_stage_of.assign(kMaxIntervals, 0);
        for (size_t i = 0; i < g_events.size(); ++i) {
            if (hipEventCreate(&g_events[i]) != hipSuccess) {
                for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(g_events[j]);
                g_events.clear();
                return FLURKA_ERR_LAUNCH;
            }
        }
        g_intervals = 0;
        g_open = false;
        g_prof_on = true;
    } else if (!on && g_prof_on) {
        g_prof_on = false;
        for (hipEvent_t e : g_events) (void)hipEventDestroy(e);
        g_events.clear();
        g_intervals = 0;
    }
    return FLURKA_OK;
}

int flurka_profile_read(int* stage_ids, float* milliseconds, int capacity) {
    if (!g_prof_on || !stage_ids || !milliseconds || capacity < 1) return 0;
    int written = 0;
    for (int i = 0; i < g_intervals && written < capacity; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_events[2 * i + 1]) != hipSuccess) break;
        if (hipEventElapsedTime(&ms, g_events[2 * i], g_events[2 * i + 1]) != hipSuccess) break;
        stage_ids[written] = g_stage_of[i];
        milliseconds[written] = ms;
        ++written;
    }
    g_intervals = 0;
    g_open = false;
    return written;
}

const char* flurka_profile_stage_name(int id) {
    switch (id) {
        case STAGE_PROJECT: return "project";
        case STAGE_KEY_STATE: return "key_state";
        case STAGE_QUERY: return "query_stream";
        case STAGE_BWD_QUERY: return "bwd_query";
        case STAGE_BWD_KEY: return "bwd_key";
        case STAGE_BWD_DKDV: return "bwd_dk_dv";
        case STAGE_BWD_DEDF: return "bwd_de_df";
        case STAGE_K_PROJ_GEMM: return "project:gemm_mfma_proj";
        case STAGE_K_PROJ_FINISH: return "project:proj_finish";
        case STAGE_K_KEY_STATE: return "key_state:key_state";
        case STAGE_K_MERGE_PACK: return "key_state:merge_pack";
        case STAGE_K_QUERY_STREAM: return "query_stream:query_stream";
        case STAGE_K_BWD_X: return "bwd_query:bwd_query_x";
        case STAGE_K_BWD_Y: return "bwd_query:bwd_query_y";
        case STAGE_K_BWD_MERGE: return "bwd_key:bwd_merge";
        case STAGE_K_BWD_KEY: return "bwd_key:bwd_key";
        case STAGE_K_GRAD_X: return "bwd_dk_dv:gemm_mfma_gradx";
        case STAGE_K_GRAD_E: return "bwd_de_df:gemm_mfma_grade";
        case STAGE_K_SUM_SPLITS: return "bwd_grad_gemms:sum_splits";
        case STAGE_BWD_GRADS: return "bwd_grad_gemms";
        case STAGE_K_GRAD_PAIR: return "bwd_grad_gemms:gemm_mfma_grads";
        case STAGE_K_WIDE_GEMM: return "project:gemm_mfma_wide";
        case STAGE_K_WIDE_FINISH: return "project:wide_finish";
        case STAGE_K_TRANSFORM_GEMM: return "project:gemm_mfma_transform";
        case STAGE_K_IDENTITY_PACK: return "key_state:identity_pack";
        case STAGE_K_LINFORMER_PACK: return "key_state:linformer_pack";
    }
    return "unknown";
}

}  // extern "C"
