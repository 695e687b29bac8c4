// Eigendecomposition of C = G^T G, the cutoff j and the coefficient vector c
// (Section 2: Sigma_G / V_G, the rule after eq. (3), alpha_k of eq. (4)).
//
// One workgroup, everything in LDS, fp64 throughout.  The solver is the
// parallel-order two-sided Jacobi method: the m indices are paired by a
// round-robin tournament (m/2 disjoint pairs per round, m-1 rounds per sweep);
// in each round the m/2 plane rotations are computed first, then every 2x2
// block of the matrix (pair x pair) is updated as J_a^T B J_b by one thread, and
// the eigenvector matrix is updated as V J.  Odd m is padded with an inert zero
// row/column.
#include "qn_internal.h"

namespace qn {

constexpr int kEigThreads = 256;
constexpr int kEigMaxSweeps = 30;
constexpr int kLd = QN_MAX_M + 1;   // padded leading dimension in LDS

__device__ __forceinline__ double block_sum(double v, double *scratch)
{
    // fixed-order tree over the workgroup
    scratch[threadIdx.x] = v;
    __syncthreads();
    for (int s = kEigThreads / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s)
            scratch[threadIdx.x] += scratch[threadIdx.x + s];
        __syncthreads();
    }
    const double r = scratch[0];
    __syncthreads();
    return r;
}

__global__ __launch_bounds__(kEigThreads) void eig_select(
    const double *__restrict__ C, const double *__restrict__ w, int m,
    double lambda, double *__restrict__ sigma_out, double *__restrict__ V_out,
    float *__restrict__ c_out, int *__restrict__ j_out)
{
    __shared__ double A[QN_MAX_M][kLd];
    __shared__ double V[QN_MAX_M][kLd];      // V[k][r]: component r of column k
    __shared__ double scratch[kEigThreads];
    __shared__ double cs[QN_MAX_M / 2], sn[QN_MAX_M / 2];
    __shared__ int pp[QN_MAX_M / 2], qq[QN_MAX_M / 2];
    __shared__ double wv[QN_MAX_M], sig[QN_MAX_M], coef[QN_MAX_M], cvec[QN_MAX_M];
    __shared__ int perm[QN_MAX_M];
    __shared__ int bad, jsel;

    const int tid = threadIdx.x;
    const int M = m + (m & 1);
    if (tid == 0)
        bad = 0;
    __syncthreads();

    // load the symmetric part; pad; V = I; non-finite scan
    for (int e = tid; e < QN_MAX_M * QN_MAX_M; e += kEigThreads) {
        const int k = e / QN_MAX_M, l = e % QN_MAX_M;
        double v = 0.0;
        if (k < m && l < m) {
            v = 0.5 * (C[l * m + k] + C[k * m + l]);
            if (!isfinite(v))
                bad = 1;
        }
        A[k][l] = v;
        V[k][l] = (k == l) ? 1.0 : 0.0;
    }
    if (tid < m) {
        wv[tid] = w[tid];
        if (!isfinite(wv[tid]))
            bad = 1;
    }
    __syncthreads();

    if (bad) {   // uniform: read after the barrier
        if (tid < m) {
            c_out[tid] = 0.0f;
            if (sigma_out)
                sigma_out[tid] = __longlong_as_double(0x7ff8000000000000LL);
        }
        if (V_out)
            for (int e = tid; e < m * m; e += kEigThreads)
                V_out[e] = __longlong_as_double(0x7ff8000000000000LL);
        if (tid == 0)
            *j_out = -1;
        return;
    }

    double tot = 0.0;
    for (int e = tid; e < M * M; e += kEigThreads) {
        const double v = A[e / M][e % M];
        tot += v * v;
    }
    const double total2 = block_sum(tot, scratch);
    const double tol2 = 1e-28 * total2;

    const int npairs = M / 2;
    for (int sweep = 0; sweep < kEigMaxSweeps; ++sweep) {
        double off = 0.0;
        for (int e = tid; e < M * M; e += kEigThreads) {
            const int k = e / M, l = e % M;
            if (k != l)
                off += A[k][l] * A[k][l];
        }
        const double off2 = block_sum(off, scratch);
        if (off2 <= tol2)
            break;

        for (int round = 0; round < M - 1; ++round) {
            if (tid < npairs) {
                int p, q;
                if (tid == 0) {
                    p = round;
                    q = M - 1;
                } else {
                    p = (round + tid) % (M - 1);
                    q = (round - tid + (M - 1)) % (M - 1);
                }
                if (p > q) {
                    const int t = p;
                    p = q;
                    q = t;
                }
                const double apq = A[p][q];
                double c = 1.0, s = 0.0;
                if (apq != 0.0) {
                    const double zeta = (A[q][q] - A[p][p]) / (2.0 * apq);
                    const double t = copysign(1.0, zeta) /
                                     (fabs(zeta) + sqrt(zeta * zeta + 1.0));
                    c = 1.0 / sqrt(t * t + 1.0);
                    s = t * c;
                }
                pp[tid] = p;
                qq[tid] = q;
                cs[tid] = c;
                sn[tid] = s;
            }
            __syncthreads();
            // A <- J^T A J, one 2x2 block (pair a) x (pair b) per thread
            for (int blk = tid; blk < npairs * npairs; blk += kEigThreads) {
                const int a = blk / npairs, b = blk % npairs;
                const int p1 = pp[a], q1 = qq[a], p2 = pp[b], q2 = qq[b];
                const double c1 = cs[a], s1 = sn[a], c2 = cs[b], s2 = sn[b];
                const double b00 = A[p1][p2], b01 = A[p1][q2];
                const double b10 = A[q1][p2], b11 = A[q1][q2];
                const double t00 = c1 * b00 - s1 * b10, t01 = c1 * b01 - s1 * b11;
                const double t10 = s1 * b00 + c1 * b10, t11 = s1 * b01 + c1 * b11;
                double n00 = c2 * t00 - s2 * t01, n01 = s2 * t00 + c2 * t01;
                double n10 = c2 * t10 - s2 * t11, n11 = s2 * t10 + c2 * t11;
                if (a == b) {   // the annihilated pair: exactly diagonal
                    n01 = 0.0;
                    n10 = 0.0;
                }
                A[p1][p2] = n00;
                A[p1][q2] = n01;
                A[q1][p2] = n10;
                A[q1][q2] = n11;
            }
            // V <- V J
            for (int it = tid; it < npairs * M; it += kEigThreads) {
                const int a = it / M, r = it % M;
                const int p = pp[a], q = qq[a];
                const double c = cs[a], s = sn[a];
                const double vp = V[p][r], vq = V[q][r];
                V[p][r] = c * vp - s * vq;
                V[q][r] = s * vp + c * vq;
            }
            __syncthreads();
        }
    }

    // sort descending by counting; sigma = sqrt(max(mu, 0))
    if (tid < m) {
        const double mu = A[tid][tid];
        int rank = 0;
        for (int l = 0; l < m; ++l) {
            const double ml = A[l][l];
            rank += (ml > mu) || (ml == mu && l < tid);
        }
        perm[rank] = tid;
        sig[rank] = mu > 0.0 ? sqrt(mu) : 0.0;
    }
    __syncthreads();

    // cutoff: number of sigma_k >= lambda * sigma_1 (sigma is sorted)
    if (tid == 0) {
        int j = 0;
        if (sig[0] > 0.0) {
            const double thr = lambda * sig[0];
            while (j < m && sig[j] >= thr)
                ++j;
        }
        jsel = j;
        *j_out = j;
    }
    __syncthreads();
    const int j = jsel;

    // alpha_k = v_k^T w / sigma_k ; coef_k = alpha_k / sigma_k
    if (tid < m) {
        double cf = 0.0;
        if (tid < j) {
            const int col = perm[tid];
            double dot = 0.0;
            for (int r = 0; r < m; ++r)
                dot += V[col][r] * wv[r];
            cf = (dot / sig[tid]) / sig[tid];
        }
        coef[tid] = cf;
    }
    __syncthreads();
    if (tid < m) {
        double s = 0.0;
        for (int k = 0; k < j; ++k)
            s += V[perm[k]][tid] * coef[k];
        cvec[tid] = s;
    }
    __syncthreads();
    if (tid < m) {
        // 1^T c = 0 in exact arithmetic (every kept v_k is orthogonal to the
        // all-ones null vector); remove the rounding residue
        double mean = 0.0;
        for (int r = 0; r < m; ++r)
            mean += cvec[r];
        mean /= m;
        c_out[tid] = static_cast<float>(cvec[tid] - mean);
        if (sigma_out)
            sigma_out[tid] = sig[tid];
    }
    if (V_out)
        for (int e = tid; e < m * m; e += kEigThreads) {
            const int k = e / m, r = e % m;
            V_out[e] = V[perm[k]][r];
        }
}

int launch_eig(const double *C, const double *w, int m, float lambda,
               double *sigma, double *V, float *c, int *j_out,
               hipStream_t stream)
{
    TraceScope ts(QN_K_EIG, stream);
    hipLaunchKernelGGL(eig_select, dim3(1), dim3(kEigThreads), 0, stream, C, w, m,
                       static_cast<double>(lambda), sigma, V, c, j_out);
    return check_launch();
}

}  // namespace qn
