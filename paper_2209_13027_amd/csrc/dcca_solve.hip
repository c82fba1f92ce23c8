// DCCA solve (Eq. 2-3) in one workgroup, fp64, matrices resident in LDS:
//   B_d = C_dd + eps_d I (ridge), C~ = 2 C_w - C_T
//   B_d = L_d L_d^T (Cholesky), L_d^{-1} formed in place, T = L_1^{-1} C~ L_2^{-T}
//   T = Q R by modified Gram-Schmidt (one barrier per column; only R is kept), then R^T = Z diag(sigma) W^T
//   by one-sided (Hestenes) Jacobi rotations of column pairs of R^T in round-robin order, one 8-lane group
//   per pair, one barrier per round.  The triangular factor takes a third fewer sweeps than T itself on the
//   graded matrices of image patches, and T = (Q W) diag(sigma) Z^T: the right singular vectors v of T are
//   the normalised columns the rotations end with, u = T v / sigma for the L leading triplets only
//   w_1 = L_1^{-T} u,  w_2 = L_2^{-T} v,  rho = sigma
// The leading L pairs are written as fp32 filters (Eq. 4-5: row-major k x k).
#include "ddcca_internal.h"

namespace ddcca {

constexpr int SOLVE_THREADS = 1024;
constexpr int SOLVE_MAX_SWEEPS = 40;
constexpr double SOLVE_TOL = 1e-15;      // rotate while |g_p . g_q| > tol * |g_p| |g_q|
constexpr double SOLVE_QUAD = 1e-5;      // a sweep whose largest cosine was below this is the last one

struct SolveParams {
    const double *C11, *C22, *Cw, *CT;
    int L;
    double ridge;
    double *gI1, *gI2;          // global scratch: the two inverse Cholesky factors
    float *W1, *W2;
    double *rho;
    int *flags;                 // device int[4]: [0] bad class label seen during the accumulation (read: the
                                // outputs are then NaN), [1] a Cholesky pivot was not positive and finite,
                                // [2] the rotations did not converge within SOLVE_MAX_SWEEPS (both written)
};

// Sum over the 16 lanes of a DPP row (lanes 16r .. 16r+15), result in every lane of the row.
// Rotations by 8, 4, 2, 1 within the row; every lane ends with bit-identical totals.
__device__ __forceinline__ double row16_sum(double x)
{
#define DDCCA_ROR(n)                                                                                   \
    {                                                                                                  \
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), 0x120 + (n), 0xf, 0xf, false); \
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), 0x120 + (n), 0xf, 0xf, false); \
        x += __hiloint2double(hi, lo);                                                                 \
    }
    DDCCA_ROR(8) DDCCA_ROR(4) DDCCA_ROR(2) DDCCA_ROR(1)
#undef DDCCA_ROR
    return x;
}

// max over the 16 lanes of a DPP row, result in every lane.
__device__ __forceinline__ double row16_max(double x)
{
#define DDCCA_ROR(n)                                                                                   \
    {                                                                                                  \
        const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), 0x120 + (n), 0xf, 0xf, false); \
        const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), 0x120 + (n), 0xf, 0xf, false); \
        x = fmax(x, __hiloint2double(hi, lo));                                                         \
    }
    DDCCA_ROR(8) DDCCA_ROR(4) DDCCA_ROR(2) DDCCA_ROR(1)
#undef DDCCA_ROR
    return x;
}

__device__ __forceinline__ int row16_min_int(int x)
{
#define DDCCA_ROR(n) x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x120 + (n), 0xf, 0xf, false));
    DDCCA_ROR(8) DDCCA_ROR(4) DDCCA_ROR(2) DDCCA_ROR(1)
#undef DDCCA_ROR
    return x;
}


// One lane-exchange step of a double: both halves through the data-parallel primitive `ctrl`.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x)
{
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// Sums of a, b, c over the 8 lanes of a group (lanes 8r .. 8r+7), results in every lane of the group and
// bit-identical there.  Exchanges: lane^1, lane^2 (quad permutations), 7-lane (mirror of the half row).  The
// three sums advance in lockstep so that their dependent chains overlap.
__device__ __forceinline__ void group8_sum3(double &a, double &b, double &c)
{
#define DDCCA_STEP(ctrl)                                                                     \
    {                                                                                        \
        const double ta = dpp_f64<ctrl>(a), tb = dpp_f64<ctrl>(b), tc = dpp_f64<ctrl>(c);    \
        a += ta;                                                                             \
        b += tb;                                                                             \
        c += tc;                                                                             \
    }
    DDCCA_STEP(0xb1) DDCCA_STEP(0x4e) DDCCA_STEP(0x141)
#undef DDCCA_STEP
}

// 1/sqrt(x) to fp64 accuracy for normal positive x: hardware estimate + two Newton steps.
__device__ __forceinline__ double fast_rsqrt(double x)
{
    double y = __builtin_amdgcn_rsq(x);
    y = y * (1.5 - 0.5 * x * y * y);
    y = y * (1.5 - 0.5 * x * y * y);
    return y;
}

template <int KS>
__global__ __launch_bounds__(SOLVE_THREADS) void dcca_solve_kernel(SolveParams p)
{
    extern __shared__ double sm[];
    constexpr int D = KS * KS, DD = D * D;
    constexpr int NR = (D + 15) / 16;            // rows of a column held by one lane of a 16-lane group
    constexpr int NGRP = SOLVE_THREADS / 16;
    constexpr int GPASS = (D - 1 + NGRP - 1) / NGRP;   // passes of the groups over up to D-1 filter pairs
    const int L = p.L;
    double *A = sm, *B = sm + DD, *C = sm + 2 * DD;
    double *small = sm + 3 * DD;                 // [2*D + 8] doubles
    double *lam = small;                         // D
    double *red = small + D;                     // 8
    int *ip = reinterpret_cast<int *>(small + 2 * D + 8);   // [D + 4] ints
    int *order = ip, *flag = ip + D;
    const int tid = threadIdx.x, nt = SOLVE_THREADS;
    const int grp = tid >> 4, l16 = tid & 15;
    const bool poisoned = p.flags[0] != 0;

    // ---- load, symmetrise, ridge -----------------------------------------------------
    for (int e = tid; e < DD; e += nt) {
        const int i = e / D, j = e - i * D;
        A[e] = 0.5 * (p.C11[e] + p.C11[j * D + i]);
        B[e] = 0.5 * (p.C22[e] + p.C22[j * D + i]);
        C[e] = 2.0 * p.Cw[e] - p.CT[e];
    }
    __syncthreads();
    if (tid < 2) {
        const double *m = tid == 0 ? A : B;
        double tr = 0.0;
        for (int i = 0; i < D; ++i) tr += m[i * D + i];
        red[tid] = p.ridge * tr / D;
    }
    __syncthreads();
    if (tid < D) A[tid * D + tid] += red[0];
    else if (tid < 2 * D) B[(tid - D) * D + (tid - D)] += red[1];
    __syncthreads();

    // ---- Cholesky of both matrices (lower factor, in place), half of the workgroup each;
    //      a half is 32 row-groups of 16 lanes ---------------------------------------------
    {
        constexpr int half = SOLVE_THREADS / 2;
        double *m = tid < half ? A : B;
        const int t = tid < half ? tid : tid - half;
        const int ty = t >> 4, tx = t & 15;
        for (int j = 0; j < D; ++j) {
            const double piv = m[j * D + j];
            if (t == 0 && !(piv > 0.0 && piv <= 1.7976931348623157e308)) p.flags[1] = 1;
            const double rd = fast_rsqrt(piv);
            for (int i = j + 1 + t; i < D; i += half) m[i * D + j] *= rd;
            __syncthreads();
            if (t == 0) m[j * D + j] = piv * rd;
            for (int i = j + 1 + ty; i < D; i += 32) {
                const double lij = m[i * D + j];
                for (int c = j + 1 + tx; c <= i; c += 16) m[i * D + c] -= lij * m[c * D + j];
            }
            __syncthreads();
        }
        // ---- in-place inverse of the lower factor, last column first: with the trailing block
        //      already inverted, column j of the inverse is -(1/l_jj) * Linv[j+1:, j+1:] * l[j+1:, j]
        constexpr int RP = (D + 31) / 32;
        for (int j = D - 1; j >= 0; --j) {
            const double ajj = 1.0 / m[j * D + j];
            double tmp[RP];
#pragma unroll
            for (int r = 0; r < RP; ++r) {
                const int i = j + 1 + ty + 32 * r;
                double s = 0.0;
                if (i < D)
                    for (int c = j + 1 + tx; c <= i; c += 16) s += m[i * D + c] * m[c * D + j];
                tmp[r] = row16_sum(s);
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < RP; ++r) {
                const int i = j + 1 + ty + 32 * r;
                if (i < D && tx == 0) m[i * D + j] = -ajj * tmp[r];
            }
            if (t == 0) m[j * D + j] = ajj;
            __syncthreads();
        }
    }
    // ---- T = L1^{-1} C~ L2^{-T}:  X = A*C -> B (B saved to global first), T = X * inv2^T -> C
    for (int e = tid; e < DD; e += nt) p.gI2[e] = B[e];
    __syncthreads();
    for (int e = tid; e < DD; e += nt) {
        const int i = e / D, c = e - i * D;
        double s = 0.0;
        for (int j = 0; j <= i; ++j) s += A[i * D + j] * C[j * D + c];
        B[e] = s;
    }
    for (int e = tid; e < DD; e += nt) p.gI1[e] = A[e];
    __syncthreads();
    for (int e = tid; e < DD; e += nt) A[e] = p.gI2[e];
    __syncthreads();
    for (int e = tid; e < DD; e += nt) {
        const int i = e / D, c = e - i * D;
        double s = 0.0;
        for (int j = 0; j <= c; ++j) s += B[i * D + j] * A[c * D + j];
        C[e] = s;
    }
    __syncthreads();

    // ---- A <- T^T (one column of T per row)
    for (int e = tid; e < DD; e += nt) {
        const int pcol = e / D, i = e - pcol * D;
        A[e] = C[i * D + pcol];
    }
    // ---- T = Q R by modified Gram-Schmidt on the columns of T (rows of A); row j of R goes to row j of B.
    //      Step j: every later column i takes r_ji = a_j . a_i / |a_j| and drops its component along a_j; a_j
    //      itself is only read, so one barrier per step is enough.
    for (int e = tid; e < DD; e += nt) B[e] = 0.0;
    __syncthreads();
    {
        constexpr int MR = (D + 7) / 8, NG8 = SOLVE_THREADS / 8;
        const int g8 = tid >> 3, m8 = tid & 7;
        for (int j = 0; j < D; ++j) {
            for (int i = j + g8; i < D; i += NG8) {
                const double *aj = A + j * D;
                double *ai = A + i * D;
                double xj[MR], xi[MR];
                double dj = 0.0, di = 0.0, unused = 0.0;
#pragma unroll
                for (int r = 0; r < MR; ++r) {
                    const int e = m8 + 8 * r;
                    xj[r] = e < D ? aj[e] : 0.0;
                    xi[r] = e < D ? ai[e] : 0.0;
                    dj += xj[r] * xj[r];
                    di += xj[r] * xi[r];
                }
                group8_sum3(dj, di, unused);
                const double rinv = dj > 0.0 ? fast_rsqrt(dj) : 0.0;
                if (i == j) {
                    if (m8 == 0) B[j * D + j] = dj * rinv;
                } else {
                    const double rji = di * rinv, coef = rji * rinv;
#pragma unroll
                    for (int r = 0; r < MR; ++r) {
                        const int e = m8 + 8 * r;
                        if (e < D) ai[e] = xi[r] - coef * xj[r];
                    }
                    if (m8 == 0) B[j * D + i] = rji;
                }
            }
            __syncthreads();
        }
    }
    double *const J = B;                          // the rotations work on the rows of B = columns of R^T
    if (tid == 0) flag[0] = 0;
    __syncthreads();

    // A group of 8 lanes owns one column pair per round: it forms the three inner products and
    // the rotation that makes the two columns orthogonal, and applies it.  Pairs of one round
    // are disjoint (round-robin tournament), so a round needs a single barrier.  Eight lanes per
    // pair put all pairs of a round into at most one wavefront per SIMD up to k = 7.
    constexpr int NP = D + (D & 1);              // players; index D (if present) is a bye
    constexpr int N_PAIRS = NP / 2, N_ROUNDS = NP - 1;
    constexpr int JR = (D + 7) / 8;              // rows of a column held by one lane of the group
    static_assert(N_PAIRS <= SOLVE_THREADS / 8, "one 8-lane group per pair");
    const int jg = tid >> 3, l8 = tid & 7;
    int coarse = 1;
    for (int sweep = 0; sweep < SOLVE_MAX_SWEEPS; ++sweep) {
        for (int round = 0; round < N_ROUNDS; ++round) {
            if (jg < N_PAIRS) {
                int a, b;
                if (jg == 0) {
                    a = NP - 1;
                    b = round;
                } else {
                    a = round + jg;
                    if (a >= NP - 1) a -= NP - 1;
                    b = round - jg;
                    if (b < 0) b += NP - 1;
                }
                const int pp = min(a, b), qq = max(a, b);
                if (qq < D) {
                    double *gp = J + pp * D, *gq = J + qq * D;
                    double x[JR], y[JR];
#pragma unroll
                    for (int r = 0; r < JR; ++r) {
                        const int i = l8 + 8 * r;
                        const bool in = i < D;
                        x[r] = in ? gp[i] : 0.0;
                        y[r] = in ? gq[i] : 0.0;
                    }
                    double al = 0.0, be = 0.0, ga = 0.0;
#pragma unroll
                    for (int r = 0; r < JR; ++r) {
                        al += x[r] * x[r];
                        be += y[r] * y[r];
                        ga += x[r] * y[r];
                    }
                    group8_sum3(al, be, ga);
                    if (ga * ga > (SOLVE_TOL * SOLVE_TOL) * (al * be)) {
                        // rotation angle theta, |theta| <= pi/4, tan(2 theta) = 2 ga / (be - al):
                        // cos(2 theta) = |d|/r, c = sqrt((1 + cos 2theta)/2), s = sin(2 theta)/(2c)
                        const double d = be - al, g2 = 2.0 * ga;
                        const double rinv = fast_rsqrt(d * d + g2 * g2);
                        const double h = 0.5 + 0.5 * fabs(d) * rinv;       // c^2, in [0.5, 1]
                        const double cinv = fast_rsqrt(h);
                        const double c = h * cinv;
                        const double sn = (d >= 0.0 ? 0.5 : -0.5) * g2 * rinv * cinv;
#pragma unroll
                        for (int r = 0; r < JR; ++r) {
                            const int i = l8 + 8 * r;
                            if (i < D) {
                                gp[i] = c * x[r] - sn * y[r];
                                gq[i] = sn * x[r] + c * y[r];
                            }
                        }
                        // was any pair of this sweep further from orthogonal than SOLVE_QUAD ?
                        if (l8 == 0 && ga * ga > (SOLVE_QUAD * SOLVE_QUAD) * (al * be)) flag[0] = 1;
                    }
                }
            }
            __syncthreads();
        }
        coarse = flag[0];
        __syncthreads();
        if (tid == 0) flag[0] = 0;
        __syncthreads();
        // Cyclic Jacobi converges quadratically: once every pair of a sweep was orthogonal to
        // SOLVE_QUAD (cosine), the rotations of that sweep leave cosines of order SOLVE_QUAD^2.
        if (!coarse) break;
    }
    if (coarse && tid == 0) p.flags[2] = 1;

    // ---- squared singular values = squared column norms; order them (descending, index breaks ties)
    for (int col = grp; col < D; col += NGRP) {
        const double *gp = J + col * D;
        double al = 0.0;
        for (int i = l16; i < D; i += 16) al += gp[i] * gp[i];
        al = row16_sum(al);
        if (l16 == 0) lam[col] = al;
    }
    __syncthreads();
    if (tid < D) {
        const double me = lam[tid];
        int rank = 0;
        for (int j = 0; j < D; ++j) {
            const double o = lam[j];
            if (o > me || (o == me && j < tid)) ++rank;
        }
        order[rank] = tid;
    }
    __syncthreads();

    // ---- v_g = (column j of the rotated R^T) / sigma_j into A[g][:];  u_g = T v_g (unscaled) into B[g][:]
    for (int e = tid; e < L * D; e += nt) {
        const int g = e / D, i = e - g * D;
        const int j = order[g];
        const double l2 = lam[j];
        A[e] = l2 > 0.0 ? J[j * D + i] * fast_rsqrt(l2) : 0.0;
    }
    __syncthreads();
    for (int e = tid; e < L * D; e += nt) {
        const int g = e / D, i = e - g * D;
        double s = 0.0;
        for (int c = 0; c < D; ++c) s += C[i * D + c] * A[g * D + c];
        B[e] = s;                                   // scaled to unit length below
    }
    __syncthreads();
    // ---- w1 = L1^{-T} u, u normalised to unit length: one 16-lane group per pair g; sign from the
    //      largest-magnitude entry
    for (int e = tid; e < DD; e += nt) C[e] = p.gI1[e];
    __syncthreads();
    double sign_of[GPASS];
#pragma unroll
    for (int pass = 0; pass < GPASS; ++pass) {
        const int g = grp + pass * NGRP;
        double sg = 1.0;
        if (g < L) {
            const double *u = B + g * D;
            double nu = 0.0;
            for (int i = l16; i < D; i += 16) nu += u[i] * u[i];
            nu = row16_sum(nu);
            const double scale = nu > 0.0 ? fast_rsqrt(nu) : 0.0;
            double w[NR];
            double best = -1.0;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int i = l16 + 16 * r;
                double s = 0.0;
                if (i < D)
                    for (int j = i; j < D; ++j) s += C[j * D + i] * u[j];
                w[r] = scale * s;
                if (i < D) best = fmax(best, fabs(w[r]));
            }
            const double top = row16_max(best);
            int arg = 1 << 30;
#pragma unroll
            for (int r = NR - 1; r >= 0; --r) {
                const int i = l16 + 16 * r;
                if (i < D && fabs(w[r]) == top) arg = i;
            }
            arg = row16_min_int(arg);               // lowest index among ties
            double neg = 0.0;
#pragma unroll
            for (int r = 0; r < NR; ++r)
                if (l16 + 16 * r == arg && w[r] < 0.0) neg = 1.0;
            neg = row16_max(neg);
            sg = neg > 0.0 ? -1.0 : 1.0;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int i = l16 + 16 * r;
                if (i < D) p.W1[g * D + i] = poisoned ? __builtin_nanf("") : (float)(sg * w[r]);
            }
            if (l16 == 0) {
                const double l2 = lam[order[g]];
                p.rho[g] = poisoned ? __builtin_nan("") : l2 > 0.0 ? sqrt(l2) : 0.0;
            }
        }
        sign_of[pass] = sg;
    }
    __syncthreads();
    // ---- w2 = L2^{-T} v (v has unit length), same sign ------------------------------------------
    for (int e = tid; e < DD; e += nt) C[e] = p.gI2[e];
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < GPASS; ++pass) {
        const int g = grp + pass * NGRP;
        if (g < L) {
            const double *v = A + g * D;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int i = l16 + 16 * r;
                if (i < D) {
                    double s = 0.0;
                    for (int j = i; j < D; ++j) s += C[j * D + i] * v[j];
                    p.W2[g * D + i] = poisoned ? __builtin_nanf("") : (float)(sign_of[pass] * s);
                }
            }
        }
    }
}

template <int KS>
static int solve_launch(ddcca_ctx *ctx, const SolveParams &p)
{
    constexpr int D = KS * KS;
    const size_t lds = (size_t)(3 * D * D + 2 * D + 8) * sizeof(double) + (size_t)(D + 4) * sizeof(int);
    static bool attr_set[MAX_DEVICES] = {};      // the attribute belongs to the kernel's code object on ONE device
    if (!attr_set[ctx->device]) {
        DDCCA_HIP(ctx, hipFuncSetAttribute((const void *)dcca_solve_kernel<KS>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(dcca_solve_kernel<KS>, dim3(1), dim3(SOLVE_THREADS), lds, ctx->stream, p);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

// ws: 2*D*D doubles of device scratch (the two inverse Cholesky factors); flags: device int[4]
static int solve_with(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw, const double *CT, int k,
                      int L, double ridge, float *W1, float *W2, double *rho, double *ws, int *flags)
{
    const int D = k * k;
    SolveParams p;
    p.C11 = C11; p.C22 = C22; p.Cw = Cw; p.CT = CT;
    p.L = L; p.ridge = ridge;
    p.gI1 = ws;
    p.gI2 = ws + (size_t)D * D;
    p.W1 = W1; p.W2 = W2; p.rho = rho;
    p.flags = flags;
    switch (k) {
        case 3: return solve_launch<3>(ctx, p);
        case 5: return solve_launch<5>(ctx, p);
        case 7: return solve_launch<7>(ctx, p);
        case 9: return solve_launch<9>(ctx, p);
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
}

int launch_solve(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw, const double *CT, int k,
                 int L, double ridge, float *W1, float *W2, double *rho)
{
    const int D = k * k;
    int rc;
    if ((rc = ensure(ctx, ctx->solve_ws, 2 * (size_t)D * D * sizeof(double)))) return rc;
    if ((rc = ensure_flags(ctx))) return rc;
    ProfScope prof(ctx, DDCCA_K_SOLVE);
    return solve_with(ctx, C11, C22, Cw, CT, k, L, ridge, W1, W2, rho, (double *)ctx->solve_ws.ptr,
                      (int *)ctx->flags.ptr);
}

// ---- the solve for callers that cannot allocate ------------------------------------------------------------
// The kernel's global scratch (the two inverse Cholesky factors, 2*D*D doubles) and its int[4] of sticky
// conditions live in one file-scope device array instead of context buffers.  Every GPU holds its own copy of the
// array at its own address; the name below is only the host-side handle of the symbol, so host code never passes
// it to a kernel: the address on a device comes from hipGetSymbolAddress, once per device, with that device
// current, and is kept in static_ptr[].
constexpr size_t STATIC_WS_DOUBLES = 2 * (size_t)(DDCCA_MAX_K * DDCCA_MAX_K) * (DDCCA_MAX_K * DDCCA_MAX_K);
constexpr size_t STATIC_SCRATCH_DOUBLES = STATIC_WS_DOUBLES + 2;            // + int[4]
static __device__ __align__(256) double scratch[STATIC_SCRATCH_DOUBLES];    // 104 992 bytes per GPU, zero at load
static double *static_ptr[MAX_DEVICES] = {};

static int static_scratch(ddcca_ctx *ctx, double **ws, int **flags)
{
    if (!static_ptr[ctx->device]) {
        double *ptr = nullptr;
        DDCCA_HIP(ctx, hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(ctx, DDCCA_EHIP, "hipGetSymbolAddress returned a null address for the solve scratch");
        static_ptr[ctx->device] = ptr;
    }
    *ws = static_ptr[ctx->device];
    *flags = reinterpret_cast<int *>(static_ptr[ctx->device] + STATIC_WS_DOUBLES);
    return DDCCA_OK;
}

int launch_solve_static(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw, const double *CT,
                        int k, int L, double ridge, float *W1, float *W2, double *rho)
{
    if ((size_t)2 * k * k * k * k > STATIC_WS_DOUBLES)
        return fail(ctx, DDCCA_EINVAL, "k exceeds what the static solve scratch holds (k <= 9)");
    double *ws = nullptr;
    int *flags = nullptr;
    int rc;
    if ((rc = static_scratch(ctx, &ws, &flags))) return rc;
    ctx->static_solve_used = true;
    return solve_with(ctx, C11, C22, Cw, CT, k, L, ridge, W1, W2, rho, ws, flags);
}

// The sticky conditions of the static variant on this context's device: copied to host[4]; cleared on the device
// when any is set.  Synchronous (ddcca_status only).
int static_solve_flags(ddcca_ctx *ctx, int host[4])
{
    double *ws = nullptr;
    int *flags = nullptr;
    int rc;
    if ((rc = static_scratch(ctx, &ws, &flags))) return rc;
    DDCCA_HIP(ctx, hipMemcpy(host, flags, 4 * sizeof(int), hipMemcpyDeviceToHost));
    if (host[0] || host[1] || host[2]) DDCCA_HIP(ctx, hipMemset(flags, 0, 4 * sizeof(int)));
    return DDCCA_OK;
}

}  // namespace ddcca
