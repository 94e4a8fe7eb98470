// Generic FLuRKA attention path: every contraction is a strided, batched GEMM
// with fp32 arithmetic, joined by small row-wise kernels.  It serves the fp32
// storage type, shapes the MFMA kernels do not cover, and acts as an on-device
// cross-check for them.  Math per (batch, head), following Eq. 2 with the
// App. D row normaliser:
//   K' = E K, V' = F V;  PhiK = phi(K') (shifted);  S = PhiK^T V';  z = PhiK^T 1
//   P = phi(Q) (shifted per row);  out = (P S) / (P z)
#include "flurka_internal.h"

namespace flurka {

#define FLURKA_CHECK_LAUNCH()                                   \
    do {                                                        \
        if (hipGetLastError() != hipSuccess) return FLURKA_ERR_LAUNCH; \
    } while (0)

// ---------------------------------------------------------------------------
// Strided batched GEMM, C[b,h] (M x N) (+)= A[b,h] (M x K) * B[b,h] (K x N).
// Every operand is addressed through element strides, so transposes, shared
// operands (batch stride 0) and a reduction index that runs over (batch, d)
// pairs (K = Kout * Kin with separate strides) need no copies.
// ---------------------------------------------------------------------------
struct GemmArgs {
    const void* A;
    const void* B;
    void* C;
    int M, N, K, Kin;
    long sAm, sAki, sAko, sAb, sAh;
    long sBn, sBki, sBko, sBb, sBh;
    long sCm, sCn, sCb, sCh;
    int H;
    int a_bf16, b_bf16, c_bf16;
    int accumulate;
    int a_kfast, b_kfast;
};

constexpr int GT = 64;   // output tile edge
constexpr int GK = 16;   // reduction step

__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmArgs g) {
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int tiles_n = (g.N + GT - 1) / GT;
    const int m0 = (int)(blockIdx.x / tiles_n) * GT, n0 = (int)(blockIdx.x % tiles_n) * GT;
    const int b = blockIdx.z / g.H, h = blockIdx.z % g.H;
    const long aoff = (long)b * g.sAb + (long)h * g.sAh;
    const long boff = (long)b * g.sBb + (long)h * g.sBh;
    const long coff = (long)b * g.sCb + (long)h * g.sCh;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    // this thread's four elements of the A tile and of the B tile: LDS positions (fixed) and the loads of
    // one reduction step; the loads of step k0 + GK are in flight while step k0 is being multiplied
    int a_mm[4], a_kk[4], b_nn[4], b_kk[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (g.a_kfast) { a_kk[i] = tid & 15; a_mm[i] = (tid >> 4) + 16 * i; }
        else           { a_mm[i] = tid & 63; a_kk[i] = (tid >> 6) + 4 * i; }
        if (g.b_kfast) { b_kk[i] = tid & 15; b_nn[i] = (tid >> 4) + 16 * i; }
        else           { b_nn[i] = tid & 63; b_kk[i] = (tid >> 6) + 4 * i; }
    }
    const bool one_level = g.Kin >= g.K;        // the reduction index is not a (outer, inner) pair
    // element offsets of reduction step 0 (one-level index: a step adds GK * stride)
    long pa[4], pb[4];
    bool va[4], vb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        va[i] = m0 + a_mm[i] < g.M;
        vb[i] = n0 + b_nn[i] < g.N;
        pa[i] = aoff + (long)(m0 + a_mm[i]) * g.sAm + (long)a_kk[i] * g.sAki;
        pb[i] = boff + (long)(n0 + b_nn[i]) * g.sBn + (long)b_kk[i] * g.sBki;
    }
    float ra[4], rb[4];
    auto fetch = [&](int k0) {
        if (one_level) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ra[i] = (va[i] && k0 + a_kk[i] < g.K) ? load_elem(g.A, pa[i] + (long)k0 * g.sAki, g.a_bf16) : 0.f;
                rb[i] = (vb[i] && k0 + b_kk[i] < g.K) ? load_elem(g.B, pb[i] + (long)k0 * g.sBki, g.b_bf16) : 0.f;
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int gm = m0 + a_mm[i], gk = k0 + a_kk[i];
            float v = 0.f;
            if (gm < g.M && gk < g.K) {
                const int ko = gk / g.Kin, ki = gk - ko * g.Kin;
                v = load_elem(g.A, aoff + (long)gm * g.sAm + (long)ki * g.sAki + (long)ko * g.sAko, g.a_bf16);
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int gn = n0 + b_nn[i], gk = k0 + b_kk[i];
            float v = 0.f;
            if (gn < g.N && gk < g.K) {
                const int ko = gk / g.Kin, ki = gk - ko * g.Kin;
                v = load_elem(g.B, boff + (long)gn * g.sBn + (long)ki * g.sBki + (long)ko * g.sBko, g.b_bf16);
            }
            rb[i] = v;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < g.K; k0 += GK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            As[a_kk[i]][a_mm[i]] = ra[i];
            Bs[b_kk[i]][b_nn[i]] = rb[i];
        }
        __syncthreads();
        if (k0 + GK < g.K) fetch(k0 + GK);
        // two-level summation: a 16-term partial, then one add into the running sum
        float part[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) part[i][j] = 0.f;
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float a[4], bb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bb[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) part[i][j] = fmaf(a[i], bb[j], part[i][j]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] += part[i][j];
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= g.N) continue;
            const long ci = coff + (long)gm * g.sCm + (long)gn * g.sCn;
            float v = acc[i][j];
            if (g.accumulate) v += ((const float*)g.C)[ci];
            store_elem(g.C, ci, v, g.c_bf16);
        }
    }
}

static flurka_status launch_gemm(GemmArgs g, int batches, hipStream_t s) {
    g.a_kfast = (g.sAki == 1);
    g.b_kfast = (g.sBki == 1);
    const long tiles = (long)((g.N + GT - 1) / GT) * ((g.M + GT - 1) / GT);
    dim3 grid((unsigned)tiles, 1, batches);
    hipLaunchKernelGGL(gemm_generic_kernel, grid, dim3(256), 0, s, g);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

// ---------------------------------------------------------------------------
// Row-wise kernels.  One 64-lane wavefront per row, four rows per block.
// ---------------------------------------------------------------------------
// e_rj <- e_rj - |k'_r|^2 / 2.   rows = BH*k rows of length m in e, of length d in Kp.
__global__ __launch_bounds__(256) void key_exponent_kernel(float* e, const float* Kp, long rows, int d, int m) {
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* kr = Kp + row * d;
    float sq = 0.f;
    for (int t = lane; t < d; t += 64) sq = fmaf(kr[t], kr[t], sq);
    sq = 0.5f * wave_sum(sq);
    float* er = e + row * m;
    for (int j = lane; j < m; j += 64) er[j] -= sq;
}

// c[bh, j] = max_r e[bh, r, j]: one exponent shift per feature (any positive rescaling of a
// feature's column of phi(K') is undone by the same factor on that feature of phi(Q))
__global__ void column_max_kernel(float* c, const float* e, int k, int m, long total) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const long bh = idx / m;
    const int j = (int)(idx % m);
    const float* p = e + bh * (long)k * m + j;
    float mx = -INFINITY;
    for (int r = 0; r < k; ++r) mx = fmaxf(mx, p[(long)r * m]);
    c[idx] = mx;
}

// PhiK <- exp(e - c_j)
__global__ __launch_bounds__(256) void key_exp_kernel(float* e, const float* c, long rows, int k, int m) {
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* cc = c + (row / k) * m;
    float* er = e + row * m;
    for (int j = lane; j < m; j += 64) er[j] = expf(er[j] - cc[j]);
}

__global__ void fill_f32_kernel(float* p, float v, long count) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

__device__ __forceinline__ float elu1(float x) { return x > 0.f ? x + 1.f : expf(x); }
__device__ __forceinline__ float elu1_grad(float x) { return x > 0.f ? 1.f : expf(x); }

// dst[bh, i, :] = elu(src[bh, row0 + i, :]) + 1 for i < nr.
__global__ void elu1_rows_kernel(float* dst, const void* src, int src_bf16, long total,
                                 int nr, int d, long src_rows_per_bh, int row0) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int t = (int)(idx % d);
    const long r = idx / d;
    const long bh = r / nr, i = r % nr;
    dst[idx] = elu1(load_elem(src, (bh * src_rows_per_bh + row0 + i) * d + t, src_bf16));
}

// z[bh, j] = sum_r PhiK[bh, r, j]
__global__ void column_sum_kernel(float* z, const float* Phi, int k, int m, long total) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const long bh = idx / m;
    const int j = (int)(idx % m);
    const float* p = Phi + bh * (long)k * m + j;
    float s = 0.f;
    for (int r = 0; r < k; ++r) s += p[(long)r * m];
    z[idx] = s;
}

// P[row, :] <- exp(v - max_j v), v_j = U[row, j] + c[bh, j]   (rows = BH*nr).  With `rowmax` (the
// lse segment, forward only) the maximum of row (bh, row0 + i) is left there for fwd_finish_kernel.
__global__ __launch_bounds__(256) void row_exp_kernel(float* U, const float* c, long rows, int nr, int m,
                                                      float* rowmax, int n, int row0) {
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    float* u = U + row * m;
    const float* cc = c + (row / nr) * m;
    float mx = -INFINITY;
    for (int j = lane; j < m; j += 64) mx = fmaxf(mx, u[j] + cc[j]);
    mx = wave_max(mx);
    for (int j = lane; j < m; j += 64) u[j] = expf(u[j] + cc[j] - mx);
    if (rowmax && lane == 0) rowmax[(row / nr) * n + row0 + row % nr] = mx;
}

// D = P.z ; out = N / D  (rows = BH*nr; output row = bh*n + row0 + i); lse = row maximum + ln D
// (`has_max`: row_exp_kernel left the maximum in lse; otherwise it is 0)
__global__ __launch_bounds__(256) void fwd_finish_kernel(const float* P, const float* N, const float* z,
                                                         void* out, int out_bf16, long rows, int nr,
                                                         int n, int row0, int mf, int d, float* lse,
                                                         int has_max) {
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const long bh = row / nr, i = row % nr;
    const float* p = P + row * mf;
    const float* zz = z + bh * mf;
    float D = 0.f;
    for (int j = lane; j < mf; j += 64) D = fmaf(p[j], zz[j], D);
    D = wave_sum(D);
    const float* nrow = N + row * d;
    const long o = (bh * n + row0 + i) * d;
    for (int t = lane; t < d; t += 64) store_elem(out, o + t, nrow[t] / D, out_bf16);
    if (lane == 0) {
        float* l = lse + bh * n + row0 + i;
        *l = (has_max ? *l : 0.f) + logf(D);
    }
}

// Backward row preparation:  D = P.z, out = N/D, dD = -(G.out)/D, N <- dN = G/D.
__global__ __launch_bounds__(256) void bwd_row_prep_kernel(const float* P, float* N, const float* z,
                                                           const void* G, int g_bf16, float* dD,
                                                           long rows, int nr, int n, int row0, int mf, int d) {
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const long bh = row / nr, i = row % nr;
    const float* p = P + row * mf;
    const float* zz = z + bh * mf;
    float D = 0.f;
    for (int j = lane; j < mf; j += 64) D = fmaf(p[j], zz[j], D);
    D = wave_sum(D);
    const float inv = 1.f / D;
    float* nrow = N + row * d;
    const long go = (bh * n + row0 + i) * d;
    float dot = 0.f;
    for (int t = lane; t < d; t += 64) {
        const float g = load_elem(G, go + t, g_bf16);
        dot = fmaf(g, nrow[t] * inv, dot);
        nrow[t] = g * inv;
    }
    dot = wave_sum(dot);
    if (lane == 0) dD[row] = -dot * inv;
}

// T <- dP (*) P with dP = T + dD_i z_j   (performer: dU of the query side)
__global__ void bwd_du_kernel(float* T, const float* P, const float* dD, const float* z,
                              long total, int nr, int mf) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const long row = idx / mf;
    const int j = (int)(idx % mf);
    const long bh = row / nr;
    T[idx] = (T[idx] + dD[row] * z[bh * mf + j]) * P[idx];
}

// elu1: dQ = (T + dD_i z_j) * phi'(Q)
__global__ void bwd_dq_elu_kernel(const float* T, const float* dD, const float* z, const void* Q,
                                  void* dQ, int bf16, long total, int nr, int n, int row0, int d) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const long row = idx / d;
    const int t = (int)(idx % d);
    const long bh = row / nr, i = row % nr;
    const long qi = (bh * n + row0 + i) * d + t;
    const float dP = T[idx] + dD[row] * z[bh * d + t];
    store_elem(dQ, qi, dP * elu1_grad(load_elem(Q, qi, bf16)), bf16);
}

// Key side, performer: dPhiK += dz_j; dUk = dPhiK * PhiK (in place); rs_r = sum_j dUk_rj
__global__ __launch_bounds__(256) void bwd_key_du_kernel(float* dPhi, const float* Phi, const float* dz,
                                                         float* rs, long rows, int k, int m) {
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const long bh = row / k;
    float* dp = dPhi + row * m;
    const float* ph = Phi + row * m;
    const float* dzz = dz + bh * m;
    float s = 0.f;
    for (int j = lane; j < m; j += 64) {
        const float v = (dp[j] + dzz[j]) * ph[j];
        dp[j] = v;
        s += v;
    }
    s = wave_sum(s);
    if (lane == 0) rs[row] = s;
}

// dK'_r -= rs_r K'_r
__global__ void bwd_key_norm_kernel(float* dKp, const float* Kp, const float* rs, long total, int d) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    dKp[idx] -= rs[idx / d] * Kp[idx];
}

// elu1 key side: dK' = (dPhiK + dz_j) * phi'(K')
__global__ void bwd_key_elu_kernel(float* dKp, const float* dPhi, const float* dz, const float* Kp,
                                   long total, int k, int d) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const long bh = idx / ((long)k * d);
    const int t = (int)(idx % d);
    dKp[idx] = (dPhi[idx] + dz[bh * d + t]) * elu1_grad(Kp[idx]);
}

static inline dim3 grid1d(long total, int block) { return dim3((unsigned)((total + block - 1) / block)); }

// ---------------------------------------------------------------------------
// Pieces shared by forward and backward
// ---------------------------------------------------------------------------
// P (B,H,nr,mf) <- shifted phi(Q[row0 : row0+nr]);  N (B,H,nr,d) <- P S
static flurka_status query_features_and_numerator(const Problem& p, const void* Q, const void* omega,
                                                  const float* S, const float* c, float* P, float* N,
                                                  int row0, int nr, float* rowmax, hipStream_t s) {
    const long rows = (long)p.BH * nr;
    if (!p.elu) {
        GemmArgs g{};
        g.A = (const char*)Q + (size_t)row0 * p.d * (p.bf16 ? 2 : 4);
        g.B = omega; g.C = P;
        g.M = nr; g.N = p.m; g.K = p.d; g.Kin = p.d;
        g.sAm = p.d; g.sAki = 1; g.sAb = (long)p.H * p.n * p.d; g.sAh = (long)p.n * p.d;
        g.sBn = p.d; g.sBki = 1; g.sBb = 0; g.sBh = p.omega_per_head ? (long)p.m * p.d : 0;
        g.sCm = p.m; g.sCn = 1; g.sCb = (long)p.H * nr * p.m; g.sCh = (long)nr * p.m;
        g.H = p.H; g.a_bf16 = p.bf16; g.b_bf16 = p.bf16;
        flurka_status st = launch_gemm(g, p.BH, s);
        if (st != FLURKA_OK) return st;
        hipLaunchKernelGGL(row_exp_kernel, grid1d(rows, 4), dim3(256), 0, s, P, c, rows, nr, p.m, rowmax, p.n, row0);
        FLURKA_CHECK_LAUNCH();
    } else {
        const long total = rows * p.d;
        hipLaunchKernelGGL(elu1_rows_kernel, grid1d(total, 256), dim3(256), 0, s, P, Q, p.bf16, total,
                           nr, p.d, (long)p.n, row0);
        FLURKA_CHECK_LAUNCH();
    }
    GemmArgs g{};
    g.A = P; g.B = S; g.C = N;
    g.M = nr; g.N = p.d; g.K = p.mf; g.Kin = p.mf;
    g.sAm = p.mf; g.sAki = 1; g.sAb = (long)p.H * nr * p.mf; g.sAh = (long)nr * p.mf;
    g.sBn = 1; g.sBki = p.d; g.sBb = (long)p.H * p.mf * p.d; g.sBh = (long)p.mf * p.d;
    g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * nr * p.d; g.sCh = (long)nr * p.d;
    g.H = p.H;
    return launch_gemm(g, p.BH, s);
}

// K' or V' (B,H,k,d) <- E (k,n) X (B,H,n,d)
static flurka_status project(const Problem& p, const void* E, const void* X, float* Xp, hipStream_t s) {
    GemmArgs g{};
    g.A = E; g.B = X; g.C = Xp;
    g.M = p.k; g.N = p.d; g.K = p.n; g.Kin = p.n;
    g.sAm = p.n; g.sAki = 1; g.sAb = 0; g.sAh = p.ef_per_head ? (long)p.k * p.n : 0;
    g.sBn = 1; g.sBki = p.d; g.sBb = (long)p.H * p.n * p.d; g.sBh = (long)p.n * p.d;
    g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * p.k * p.d; g.sCh = (long)p.k * p.d;
    g.H = p.H; g.a_bf16 = p.bf16; g.b_bf16 = p.bf16;
    return launch_gemm(g, p.BH, s);
}

// PhiK (k x mf, shifted) from K' in ctx.  With `new_shift` the per-feature shifts c are computed
// and stored; otherwise the stored ones are reused (backward: same PhiK as the forward had).
static flurka_status key_features(const Problem& p, const void* omega, const float* Kp, float* c,
                                  float* Phi, int new_shift, hipStream_t s) {
    const long krows = (long)p.BH * p.k;
    if (!p.elu) {
        GemmArgs g{};
        g.A = Kp; g.B = omega; g.C = Phi;
        g.M = p.k; g.N = p.m; g.K = p.d; g.Kin = p.d;
        g.sAm = p.d; g.sAki = 1; g.sAb = (long)p.H * p.k * p.d; g.sAh = (long)p.k * p.d;
        g.sBn = p.d; g.sBki = 1; g.sBb = 0; g.sBh = p.omega_per_head ? (long)p.m * p.d : 0;
        g.sCm = p.m; g.sCn = 1; g.sCb = (long)p.H * p.k * p.m; g.sCh = (long)p.k * p.m;
        g.H = p.H; g.b_bf16 = p.bf16;
        flurka_status st = launch_gemm(g, p.BH, s);
        if (st != FLURKA_OK) return st;
        hipLaunchKernelGGL(key_exponent_kernel, grid1d(krows, 4), dim3(256), 0, s, Phi, Kp, krows, p.d, p.m);
        FLURKA_CHECK_LAUNCH();
        if (new_shift) {
            const long ct = (long)p.BH * p.m;
            hipLaunchKernelGGL(column_max_kernel, grid1d(ct, 256), dim3(256), 0, s, c, (const float*)Phi, p.k,
                               p.m, ct);
            FLURKA_CHECK_LAUNCH();
        }
        hipLaunchKernelGGL(key_exp_kernel, grid1d(krows, 4), dim3(256), 0, s, Phi, (const float*)c, krows,
                           p.k, p.m);
        FLURKA_CHECK_LAUNCH();
    } else {
        const long total = krows * p.d;
        hipLaunchKernelGGL(elu1_rows_kernel, grid1d(total, 256), dim3(256), 0, s, Phi, (const void*)Kp, 0,
                           total, p.k, p.d, (long)p.k, 0);
        FLURKA_CHECK_LAUNCH();
        if (new_shift) {
            const long ct = (long)p.BH * p.d;
            hipLaunchKernelGGL(fill_f32_kernel, grid1d(ct, 256), dim3(256), 0, s, c, 0.f, ct);
            FLURKA_CHECK_LAUNCH();
        }
    }
    return FLURKA_OK;
}

// PhiK, S, z, c from K', V' (in ctx)
flurka_status generic_key_state(const Problem& p, const void* omega, float* ctx, float* Phi, hipStream_t s) {
    const CtxLayout L = ctx_layout(p);
    float* Vp = ctx + L.Vp;
    float* S = ctx + L.S;
    float* z = ctx + L.z;
    flurka_status st = key_features(p, omega, ctx + L.Kp, ctx + L.c, Phi, 1, s);
    if (st != FLURKA_OK) return st;
    // S = PhiK^T V'
    GemmArgs g{};
    g.A = Phi; g.B = Vp; g.C = S;
    g.M = p.mf; g.N = p.d; g.K = p.k; g.Kin = p.k;
    g.sAm = 1; g.sAki = p.mf; g.sAb = (long)p.H * p.k * p.mf; g.sAh = (long)p.k * p.mf;
    g.sBn = 1; g.sBki = p.d; g.sBb = (long)p.H * p.k * p.d; g.sBh = (long)p.k * p.d;
    g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * p.mf * p.d; g.sCh = (long)p.mf * p.d;
    g.H = p.H;
    st = launch_gemm(g, p.BH, s);
    if (st != FLURKA_OK) return st;
    const long zt = (long)p.BH * p.mf;
    hipLaunchKernelGGL(column_sum_kernel, grid1d(zt, 256), dim3(256), 0, s, z, (const float*)Phi, p.k, p.mf, zt);
    FLURKA_CHECK_LAUNCH();
    return FLURKA_OK;
}

// ---------------------------------------------------------------------------
// Forward
// ---------------------------------------------------------------------------
flurka_status generic_forward(const Problem& p, const FwdArgs& a, hipStream_t s) {
    const CtxLayout L = ctx_layout(p);
    const GenericWs W = generic_ws_layout(p, 0);
    flurka_status st;
    {
        StageScope sc(s, STAGE_PROJECT);
        if ((st = project(p, a.E, a.K, a.ctx + L.Kp, s)) != FLURKA_OK) return st;
        if ((st = project(p, a.F, a.V, a.ctx + L.Vp, s)) != FLURKA_OK) return st;
    }
    {
        StageScope sc(s, STAGE_KEY_STATE);
        if ((st = generic_key_state(p, a.omega, a.ctx, a.ws + W.PhiK, s)) != FLURKA_OK) return st;
    }
    const int nc = generic_chunk_rows(p);
    float* P = a.ws + W.P;
    float* N = a.ws + W.N;
    StageScope sc(s, STAGE_QUERY);
    for (int row0 = 0; row0 < p.n; row0 += nc) {
        const int nr = (p.n - row0 < nc) ? (p.n - row0) : nc;
        st = query_features_and_numerator(p, a.Q, a.omega, a.ctx + L.S, a.ctx + L.c, P, N, row0, nr, a.ctx + L.lse, s);
        if (st != FLURKA_OK) return st;
        const long rows = (long)p.BH * nr;
        hipLaunchKernelGGL(fwd_finish_kernel, grid1d(rows, 4), dim3(256), 0, s, P, N, a.ctx + L.z, a.out,
                           p.bf16, rows, nr, p.n, row0, p.mf, p.d, a.ctx + L.lse, p.elu ? 0 : 1);
        FLURKA_CHECK_LAUNCH();
    }
    return FLURKA_OK;
}

// ---------------------------------------------------------------------------
// Backward (chain rule of the forward; notation as in the forward)
//   dN = G/D, dD = -(G.out)/D, dP = dN S^T + dD z^T, dS = P^T dN, dz = P^T dD
//   dPhiK = V' dS^T + 1 dz^T, dV' = PhiK dS
//   performer: dU = dphi*phi, dx = dU omega - rowsum(dU) x  (the rowsum term is
//              identically zero on the query side: out is invariant to a
//              rescaling of a row of P);  elu1: dx = dphi * phi'(x)
//   dK = E^T dK', dV = F^T dV', dE = sum_bh dK' K^T, dF = sum_bh dV' V^T
// ---------------------------------------------------------------------------
flurka_status generic_backward(const Problem& p, const BwdArgs& a, hipStream_t s) {
    return generic_backward_from(p, a, s, 0);
}

// `done` bit 0: the caller has already written dQ and left dS, dz in the workspace slots of the
// generic layout.  Bit 1: stop after the key side (dK', dV' in the workspace); the caller runs the
// four sequence-length GEMMs itself.
flurka_status generic_backward_from(const Problem& p, const BwdArgs& a, hipStream_t s, int done) {
    const int query_done = done & 1;
    const CtxLayout L = ctx_layout(p);
    const GenericWs W = generic_ws_layout(p, 1);
    const float* Kp = a.ctx + L.Kp;
    const float* Vp = a.ctx + L.Vp;
    float* Phi = a.ws + W.PhiK;
    const float* S = a.ctx + L.S;
    const float* cshift = a.ctx + L.c;
    const float* z = a.ctx + L.z;
    float* P = a.ws + W.P;
    float* T = a.ws + W.T;
    float* N = a.ws + W.N;
    float* dD = a.ws + W.dD;
    float* dS = a.ws + W.dS;
    float* dz = a.ws + W.dz;
    float* dPhi = a.ws + W.dPhiK;
    float* dKp = a.ws + W.dKp;
    float* dVp = a.ws + W.dVp;
    float* rs = a.ws + W.rs;
    const int es = p.bf16 ? 2 : 4;
    flurka_status st;
    const int nc = generic_chunk_rows(p);

    if (!query_done) stage_begin(s);
    for (int row0 = 0; row0 < p.n && !query_done; row0 += nc) {
        const int nr = (p.n - row0 < nc) ? (p.n - row0) : nc;
        const long rows = (long)p.BH * nr;
        st = query_features_and_numerator(p, a.Q, a.omega, S, cshift, P, N, row0, nr, nullptr, s);
        if (st != FLURKA_OK) return st;
        hipLaunchKernelGGL(bwd_row_prep_kernel, grid1d(rows, 4), dim3(256), 0, s, P, N, z, a.dOut, p.bf16,
                           dD, rows, nr, p.n, row0, p.mf, p.d);
        FLURKA_CHECK_LAUNCH();
        {   // T = dN S^T  (nr x mf)
            GemmArgs g{};
            g.A = N; g.B = S; g.C = T;
            g.M = nr; g.N = p.mf; g.K = p.d; g.Kin = p.d;
            g.sAm = p.d; g.sAki = 1; g.sAb = (long)p.H * nr * p.d; g.sAh = (long)nr * p.d;
            g.sBn = p.d; g.sBki = 1; g.sBb = (long)p.H * p.mf * p.d; g.sBh = (long)p.mf * p.d;
            g.sCm = p.mf; g.sCn = 1; g.sCb = (long)p.H * nr * p.mf; g.sCh = (long)nr * p.mf;
            g.H = p.H;
            if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
        }
        if (!p.elu) {
            const long total = rows * p.mf;
            hipLaunchKernelGGL(bwd_du_kernel, grid1d(total, 256), dim3(256), 0, s, T, P, dD, z, total, nr, p.mf);
            FLURKA_CHECK_LAUNCH();
            GemmArgs g{};   // dQ = dU omega
            g.A = T; g.B = a.omega; g.C = (char*)a.dQ + (size_t)row0 * p.d * es;
            g.M = nr; g.N = p.d; g.K = p.m; g.Kin = p.m;
            g.sAm = p.m; g.sAki = 1; g.sAb = (long)p.H * nr * p.m; g.sAh = (long)nr * p.m;
            g.sBn = 1; g.sBki = p.d; g.sBb = 0; g.sBh = p.omega_per_head ? (long)p.m * p.d : 0;
            g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * p.n * p.d; g.sCh = (long)p.n * p.d;
            g.H = p.H; g.b_bf16 = p.bf16; g.c_bf16 = p.bf16;
            if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
            if (a.dOmega) {
                // d omega_j (+)= sum over (batch[, head], i) of dU_ij q_i   (u_ij = omega_j . q_i - |q_i|^2/2)
                GemmArgs w{};
                w.A = T; w.B = (const char*)a.Q + (size_t)row0 * p.d * es; w.C = a.dOmega;
                w.M = p.m; w.N = p.d; w.Kin = nr;
                w.sAm = 1; w.sAki = p.m; w.sBn = 1; w.sBki = p.d; w.sCm = p.d; w.sCn = 1;
                w.b_bf16 = p.bf16; w.accumulate = row0 > 0;
                if (p.omega_per_head) {      // one result per head, reduction over (batch, i)
                    w.K = p.B * nr; w.sAko = (long)p.H * nr * p.m; w.sAh = (long)nr * p.m;
                    w.sBko = (long)p.H * p.n * p.d; w.sBh = (long)p.n * p.d; w.sCh = (long)p.m * p.d; w.H = p.H;
                    if ((st = launch_gemm(w, p.H, s)) != FLURKA_OK) return st;
                } else {                      // one result, reduction over (batch, head, i)
                    w.K = p.BH * nr; w.sAko = (long)nr * p.m; w.sBko = (long)p.n * p.d; w.H = 1;
                    if ((st = launch_gemm(w, 1, s)) != FLURKA_OK) return st;
                }
            }
        } else {
            const long total = rows * p.d;
            hipLaunchKernelGGL(bwd_dq_elu_kernel, grid1d(total, 256), dim3(256), 0, s, T, dD, z, a.Q, a.dQ,
                               p.bf16, total, nr, p.n, row0, p.d);
            FLURKA_CHECK_LAUNCH();
        }
        {   // dS (+)= P^T dN
            GemmArgs g{};
            g.A = P; g.B = N; g.C = dS;
            g.M = p.mf; g.N = p.d; g.K = nr; g.Kin = nr;
            g.sAm = 1; g.sAki = p.mf; g.sAb = (long)p.H * nr * p.mf; g.sAh = (long)nr * p.mf;
            g.sBn = 1; g.sBki = p.d; g.sBb = (long)p.H * nr * p.d; g.sBh = (long)nr * p.d;
            g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * p.mf * p.d; g.sCh = (long)p.mf * p.d;
            g.H = p.H; g.accumulate = row0 > 0;
            if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
        }
        {   // dz (+)= P^T dD
            GemmArgs g{};
            g.A = P; g.B = dD; g.C = dz;
            g.M = p.mf; g.N = 1; g.K = nr; g.Kin = nr;
            g.sAm = 1; g.sAki = p.mf; g.sAb = (long)p.H * nr * p.mf; g.sAh = (long)nr * p.mf;
            g.sBn = 0; g.sBki = 1; g.sBb = (long)p.H * nr; g.sBh = nr;
            g.sCm = 1; g.sCn = 0; g.sCb = (long)p.H * p.mf; g.sCh = p.mf;
            g.H = p.H; g.accumulate = row0 > 0;
            if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
        }
    }

    if (!query_done) stage_end(s, STAGE_BWD_QUERY);

    stage_begin(s);
    const long krows = (long)p.BH * p.k;
    // PhiK exactly as the forward had it (same K', same shifts)
    if ((st = key_features(p, a.omega, Kp, const_cast<float*>(cshift), Phi, 0, s)) != FLURKA_OK) return st;
    {   // dPhiK = V' dS^T   (k x mf)
        GemmArgs g{};
        g.A = Vp; g.B = dS; g.C = dPhi;
        g.M = p.k; g.N = p.mf; g.K = p.d; g.Kin = p.d;
        g.sAm = p.d; g.sAki = 1; g.sAb = (long)p.H * p.k * p.d; g.sAh = (long)p.k * p.d;
        g.sBn = p.d; g.sBki = 1; g.sBb = (long)p.H * p.mf * p.d; g.sBh = (long)p.mf * p.d;
        g.sCm = p.mf; g.sCn = 1; g.sCb = (long)p.H * p.k * p.mf; g.sCh = (long)p.k * p.mf;
        g.H = p.H;
        if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
    }
    {   // dV' = PhiK dS   (k x d)
        GemmArgs g{};
        g.A = Phi; g.B = dS; g.C = dVp;
        g.M = p.k; g.N = p.d; g.K = p.mf; g.Kin = p.mf;
        g.sAm = p.mf; g.sAki = 1; g.sAb = (long)p.H * p.k * p.mf; g.sAh = (long)p.k * p.mf;
        g.sBn = 1; g.sBki = p.d; g.sBb = (long)p.H * p.mf * p.d; g.sBh = (long)p.mf * p.d;
        g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * p.k * p.d; g.sCh = (long)p.k * p.d;
        g.H = p.H;
        if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
    }
    if (!p.elu) {
        hipLaunchKernelGGL(bwd_key_du_kernel, grid1d(krows, 4), dim3(256), 0, s, dPhi, Phi, dz, rs, krows,
                           p.k, p.m);
        FLURKA_CHECK_LAUNCH();
        GemmArgs g{};   // dK' = dUk omega
        g.A = dPhi; g.B = a.omega; g.C = dKp;
        g.M = p.k; g.N = p.d; g.K = p.m; g.Kin = p.m;
        g.sAm = p.m; g.sAki = 1; g.sAb = (long)p.H * p.k * p.m; g.sAh = (long)p.k * p.m;
        g.sBn = 1; g.sBki = p.d; g.sBb = 0; g.sBh = p.omega_per_head ? (long)p.m * p.d : 0;
        g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * p.k * p.d; g.sCh = (long)p.k * p.d;
        g.H = p.H; g.b_bf16 = p.bf16;
        if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
        if (a.dOmega) {
            // d omega_j += sum over (batch[, head], r) of dUk_rj k'_r
            GemmArgs w{};
            w.A = dPhi; w.B = Kp; w.C = a.dOmega;
            w.M = p.m; w.N = p.d; w.Kin = p.k;
            w.sAm = 1; w.sAki = p.m; w.sBn = 1; w.sBki = p.d; w.sCm = p.d; w.sCn = 1;
            w.accumulate = 1;
            if (p.omega_per_head) {
                w.K = p.B * p.k; w.sAko = (long)p.H * p.k * p.m; w.sAh = (long)p.k * p.m;
                w.sBko = (long)p.H * p.k * p.d; w.sBh = (long)p.k * p.d; w.sCh = (long)p.m * p.d; w.H = p.H;
                if ((st = launch_gemm(w, p.H, s)) != FLURKA_OK) return st;
            } else {
                w.K = p.BH * p.k; w.sAko = (long)p.k * p.m; w.sBko = (long)p.k * p.d; w.H = 1;
                if ((st = launch_gemm(w, 1, s)) != FLURKA_OK) return st;
            }
        }
        const long total = krows * p.d;
        hipLaunchKernelGGL(bwd_key_norm_kernel, grid1d(total, 256), dim3(256), 0, s, dKp, Kp, rs, total, p.d);
        FLURKA_CHECK_LAUNCH();
    } else {
        const long total = krows * p.d;
        hipLaunchKernelGGL(bwd_key_elu_kernel, grid1d(total, 256), dim3(256), 0, s, dKp, dPhi, dz, Kp, total,
                           p.k, p.d);
        FLURKA_CHECK_LAUNCH();
    }

    stage_end(s, STAGE_BWD_KEY);
    if (done & 2) return FLURKA_OK;

    // dK = E^T dK', dV = F^T dV'   (n x d per head)
    stage_begin(s);
    for (int which = 0; which < 2; ++which) {
        GemmArgs g{};
        g.A = which ? a.F : a.E; g.B = which ? dVp : dKp; g.C = which ? a.dV : a.dK;
        g.M = p.n; g.N = p.d; g.K = p.k; g.Kin = p.k;
        g.sAm = 1; g.sAki = p.n; g.sAb = 0; g.sAh = p.ef_per_head ? (long)p.k * p.n : 0;
        g.sBn = 1; g.sBki = p.d; g.sBb = (long)p.H * p.k * p.d; g.sBh = (long)p.k * p.d;
        g.sCm = p.d; g.sCn = 1; g.sCb = (long)p.H * p.n * p.d; g.sCh = (long)p.n * p.d;
        g.H = p.H; g.a_bf16 = p.bf16; g.c_bf16 = p.bf16;
        if ((st = launch_gemm(g, p.BH, s)) != FLURKA_OK) return st;
    }
    stage_end(s, STAGE_BWD_DKDV);
    // dE = sum_bh dK' K^T, dF = sum_bh dV' V^T   (k x n); reduction index = (bh, t)
    stage_begin(s);
    for (int which = 0; which < 2; ++which) {
        GemmArgs g{};
        g.A = which ? dVp : dKp; g.B = which ? a.V : a.K; g.C = which ? a.dF : a.dE;
        g.M = p.k; g.N = p.n; g.Kin = p.d;
        g.sAm = p.d; g.sAki = 1; g.sBn = p.d; g.sBki = 1; g.sCm = p.n; g.sCn = 1;
        g.b_bf16 = p.bf16; g.c_bf16 = p.bf16 && !p.grad_ef_f32;
        if (p.ef_per_head) {     // one (k x n) gradient per head, reduction index = (batch, t)
            g.K = p.B * p.d; g.sAko = (long)p.H * p.k * p.d; g.sAh = (long)p.k * p.d;
            g.sBko = (long)p.H * p.n * p.d; g.sBh = (long)p.n * p.d; g.sCh = (long)p.k * p.n; g.H = p.H;
            if ((st = launch_gemm(g, p.H, s)) != FLURKA_OK) return st;
        } else {                  // E, F shared: reduction index = (batch, head, t)
            g.K = p.BH * p.d; g.sAko = (long)p.k * p.d; g.sBko = (long)p.n * p.d; g.H = 1;
            if ((st = launch_gemm(g, 1, s)) != FLURKA_OK) return st;
        }
    }
    stage_end(s, STAGE_BWD_DEDF);
    return FLURKA_OK;
}

}  // namespace flurka
