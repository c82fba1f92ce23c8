// DCCA solve (Eq. 2-3) in one workgroup, fp64, matrices resident in LDS:
//   B_d = C_dd + eps_d I (ridge), C~ = 2 C_w - C_T
//   B_d = L_d L_d^T (Cholesky), T = L_1^{-1} C~ L_2^{-T}
//   T^T T = V diag(sigma^2) V^T by parallel-ordered cyclic Jacobi rotations
//   u = T v / sigma,  w_1 = L_1^{-T} u,  w_2 = L_2^{-T} v,  rho = sigma
// The leading L pairs are written as fp32 filters (Eq. 4-5: row-major k x k).
#include "ddcca_internal.h"

namespace ddcca {

constexpr int SOLVE_THREADS = 512;
constexpr int SOLVE_MAX_SWEEPS = 40;

struct SolveParams {
    const double *C11, *C22, *Cw, *CT;
    int D, L;
    double ridge;
    double *gL1, *gL2;          // global scratch: the two Cholesky factors
    float *W1, *W2;
    double *rho;
};

// One right-looking Cholesky column step on `m` (lower triangle), done by `nt` threads
// with local id `t`; caller places a barrier after each of the two phases.
__device__ inline void chol_scale(double *m, int D, int j, int t, int nt)
{
    const double d = sqrt(m[j * D + j]);
    for (int i = j + 1 + t; i < D; i += nt) m[i * D + j] /= d;
}
__device__ inline void chol_update(double *m, int D, int j, int t, int nt)
{
    // after the scale phase m[j][j] still holds the pivot; replace it by its root last
    const int rem = D - j - 1;
    for (int e = t; e < rem * rem; e += nt) {
        const int i = j + 1 + e / rem, c = j + 1 + e % rem;
        if (c <= i) m[i * D + c] -= m[i * D + j] * m[c * D + j];
    }
}

__global__ __launch_bounds__(SOLVE_THREADS) void dcca_solve_kernel(SolveParams p)
{
    extern __shared__ double sm[];
    const int D = p.D, L = p.L, DD = D * D;
    double *A = sm, *B = sm + DD, *C = sm + 2 * DD;
    double *small = sm + 3 * DD;                 // [4*D + 8]
    double *lam = small;                         // D
    double *rc = small + D;                      // rotation cosines  (<= D/2+1)
    double *rs = small + 2 * D;                  // rotation sines
    double *red = small + 3 * D;                 // reduction scratch (>= 8 + D)
    int *ip = reinterpret_cast<int *>(small + 4 * D + 8);   // [3*D + 4] ints: pair p, pair q, order
    int *pair_p = ip, *pair_q = ip + D, *order = ip + 2 * D;
    const int tid = threadIdx.x, nt = blockDim.x;

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

    // ---- Cholesky of both matrices, half of the workgroup each -----------------------
    {
        const int half = nt / 2;
        double *m = tid < half ? A : B;
        const int t = tid < half ? tid : tid - half;
        for (int j = 0; j < D; ++j) {
            chol_scale(m, D, j, t, half);
            __syncthreads();
            chol_update(m, D, j, t, half);
            if (t == 0) m[j * D + j] = sqrt(m[j * D + j]);
            __syncthreads();
        }
    }
    // keep the factors for the final back-substitutions
    for (int e = tid; e < DD; e += nt) {
        p.gL1[e] = A[e];
        p.gL2[e] = B[e];
    }

    // ---- T = L1^{-1} C~ L2^{-T}, in place in C ---------------------------------------
    if (tid < D) {                               // column tid of X = L1^{-1} C~
        const int c = tid;
        for (int i = 0; i < D; ++i) {
            double s = C[i * D + c];
            for (int j = 0; j < i; ++j) s -= A[i * D + j] * C[j * D + c];
            C[i * D + c] = s / A[i * D + i];
        }
    }
    __syncthreads();
    if (tid < D) {                               // row tid of T: L2 t^T = x^T
        const int r = tid;
        for (int i = 0; i < D; ++i) {
            double s = C[r * D + i];
            for (int j = 0; j < i; ++j) s -= B[i * D + j] * C[r * D + j];
            C[r * D + i] = s / B[i * D + i];
        }
    }
    __syncthreads();

    // ---- M = T^T T in A, V = I in B ---------------------------------------------------
    for (int e = tid; e < DD; e += nt) {
        const int a = e / D, b = e - a * D;
        if (a <= b) {
            double s = 0.0;
            for (int r = 0; r < D; ++r) s += C[r * D + a] * C[r * D + b];
            A[a * D + b] = s;
            A[b * D + a] = s;
        }
        B[e] = (a == b) ? 1.0 : 0.0;
    }
    __syncthreads();

    // ---- cyclic Jacobi with round-robin (tournament) ordering -------------------------
    const int np = D + (D & 1);                  // players; index D (if present) is a bye
    const int n_pairs = np / 2, n_rounds = np - 1;
    double fro2 = 0.0;
    for (int sweep = 0; sweep < SOLVE_MAX_SWEEPS; ++sweep) {
        // off-diagonal and total squared norms
        double off = 0.0, all = 0.0;
        for (int e = tid; e < DD; e += nt) {
            const int i = e / D, j = e - i * D;
            const double v = A[e] * A[e];
            all += v;
            if (i != j) off += v;
        }
        for (int o = 32; o > 0; o >>= 1) {
            off += __shfl_down(off, o);
            all += __shfl_down(all, o);
        }
        if ((tid & 63) == 0) {
            red[2 * (tid >> 6)] = off;
            red[2 * (tid >> 6) + 1] = all;
        }
        __syncthreads();
        off = 0.0;
        all = 0.0;
        for (int wv = 0; wv < nt / 64; ++wv) {
            off += red[2 * wv];
            all += red[2 * wv + 1];
        }
        __syncthreads();
        if (sweep == 0) fro2 = all;
        if (off <= 1e-30 * fro2) break;          // off-diagonal norm <= 1e-15 * ||M||_F

        for (int round = 0; round < n_rounds; ++round) {
            if (tid < n_pairs) {
                int a, b;
                if (tid == 0) {
                    a = np - 1;
                    b = round;
                } else {
                    a = (round + tid) % (np - 1);
                    b = (round - tid + (np - 1)) % (np - 1);
                }
                int pp = min(a, b), qq = max(a, b);
                double c = 1.0, s = 0.0;
                if (qq < D) {
                    const double apq = A[pp * D + qq];
                    if (fabs(apq) > 1e-300) {
                        const double theta = (A[qq * D + qq] - A[pp * D + pp]) / (2.0 * apq);
                        const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                        c = 1.0 / sqrt(t * t + 1.0);
                        s = t * c;
                    }
                } else {
                    pp = qq = 0;                 // bye: identity rotation on a harmless pair
                }
                pair_p[tid] = pp;
                pair_q[tid] = qq;
                rc[tid] = c;
                rs[tid] = s;
            }
            __syncthreads();
            // columns p,q of M and of V
            for (int e = tid; e < n_pairs * D * 2; e += nt) {
                const int pr = e / (2 * D), r2 = e - pr * 2 * D;
                const int pp = pair_p[pr], qq = pair_q[pr];
                if (pp == qq) continue;
                double *m = r2 < D ? A : B;
                const int i = r2 < D ? r2 : r2 - D;
                const double c = rc[pr], s = rs[pr];
                const double x = m[i * D + pp], y = m[i * D + qq];
                m[i * D + pp] = c * x - s * y;
                m[i * D + qq] = s * x + c * y;
            }
            __syncthreads();
            // rows p,q of M
            for (int e = tid; e < n_pairs * D; e += nt) {
                const int pr = e / D, j = e - pr * D;
                const int pp = pair_p[pr], qq = pair_q[pr];
                if (pp == qq) continue;
                const double c = rc[pr], s = rs[pr];
                const double x = A[pp * D + j], y = A[qq * D + j];
                A[pp * D + j] = c * x - s * y;
                A[qq * D + j] = s * x + c * y;
            }
            __syncthreads();
        }
    }

    // ---- order the eigenvalues (descending, index breaks ties) ------------------------
    if (tid < D) lam[tid] = A[tid * D + tid];
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

    // ---- u_g = T v_g / sigma_g into A[g][:], then v_g into C[g][:] ---------------------
    for (int e = tid; e < L * D; e += nt) {
        const int g = e / D, i = e - g * D;
        const int j = order[g];
        double s = 0.0;
        for (int c = 0; c < D; ++c) s += C[i * D + c] * B[c * D + j];
        A[g * D + i] = s;                       // normalised below (||T v|| = sigma)
    }
    __syncthreads();
    for (int e = tid; e < L * D; e += nt) {
        const int g = e / D, i = e - g * D;
        C[g * D + i] = B[i * D + order[g]];
    }
    __syncthreads();
    if (tid < L) {                               // unit length for u (and v, against drift)
        double nu = 0.0, nv = 0.0;
        for (int i = 0; i < D; ++i) {
            nu += A[tid * D + i] * A[tid * D + i];
            nv += C[tid * D + i] * C[tid * D + i];
        }
        nu = nu > 0.0 ? 1.0 / sqrt(nu) : 0.0;
        nv = nv > 0.0 ? 1.0 / sqrt(nv) : 0.0;
        for (int i = 0; i < D; ++i) {
            A[tid * D + i] *= nu;
            C[tid * D + i] *= nv;
        }
    }
    __syncthreads();
    // ---- w2 = L2^{-T} v (factor reloaded into B), then w1 = L1^{-T} u -------------------
    for (int e = tid; e < DD; e += nt) B[e] = p.gL2[e];
    __syncthreads();
    if (tid < L) {
        double *x = C + tid * D;
        for (int i = D - 1; i >= 0; --i) {
            double s = x[i];
            for (int j = i + 1; j < D; ++j) s -= B[j * D + i] * x[j];
            x[i] = s / B[i * D + i];
        }
    }
    __syncthreads();
    for (int e = tid; e < DD; e += nt) B[e] = p.gL1[e];
    __syncthreads();
    if (tid < L) {
        double *x = A + tid * D;
        for (int i = D - 1; i >= 0; --i) {
            double s = x[i];
            for (int j = i + 1; j < D; ++j) s -= B[j * D + i] * x[j];
            x[i] = s / B[i * D + i];
        }
        // sign: largest-magnitude entry of w1 positive, lowest index on ties
        int arg = 0;
        double best = fabs(x[0]);
        for (int i = 1; i < D; ++i)
            if (fabs(x[i]) > best) {
                best = fabs(x[i]);
                arg = i;
            }
        const double sg = x[arg] < 0.0 ? -1.0 : 1.0;
        const double *y = C + tid * D;
        for (int i = 0; i < D; ++i) {
            p.W1[tid * D + i] = (float)(sg * x[i]);
            p.W2[tid * D + i] = (float)(sg * y[i]);
        }
        const double l2 = lam[order[tid]];
        p.rho[tid] = l2 > 0.0 ? sqrt(l2) : 0.0;
    }
}

int launch_solve(ddcca_ctx *ctx, const double *C11, const double *C22, const double *Cw, const double *CT, int k,
                 int L, double ridge, float *W1, float *W2, double *rho)
{
    ProfScope prof(ctx, DDCCA_K_SOLVE);
    const int D = k * k;
    int rc;
    if ((rc = ensure(ctx, ctx->solve_ws, 2 * (size_t)D * D * sizeof(double)))) return rc;
    SolveParams p;
    p.C11 = C11; p.C22 = C22; p.Cw = Cw; p.CT = CT;
    p.D = D; p.L = L; p.ridge = ridge;
    p.gL1 = (double *)ctx->solve_ws.ptr;
    p.gL2 = p.gL1 + (size_t)D * D;
    p.W1 = W1; p.W2 = W2; p.rho = rho;
    const size_t lds = (size_t)(3 * D * D + 4 * D + 8) * sizeof(double) + (size_t)(3 * D + 4) * sizeof(int);
    static bool attr_set = false;
    if (!attr_set) {
        DDCCA_HIP(ctx, hipFuncSetAttribute((const void *)dcca_solve_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           160 * 1024));
        attr_set = true;
    }
    hipLaunchKernelGGL(dcca_solve_kernel, dim3(1), dim3(SOLVE_THREADS), lds, ctx->stream, p);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
