// Eigendecomposition of C = G^T G, the cutoff j and the coefficient vector c
// (Section 2: Sigma_G / V_G, the rule after eq. (3), alpha_k of eq. (4)).
//
// One workgroup, everything in LDS, fp64 throughout.  The solver is the
// parallel-order two-sided Jacobi method.  The matrix is padded to M = 2, 4, 8,
// 16, 24, 32, 48 or 64 (inert zero rows/columns); the block has 256 threads (512
// at M = 48), each taking one or several of the (M/2)^2 blocks of a round.  The M indices are paired by a
// round-robin tournament: M/2 disjoint pairs per round, M-1 rounds per sweep,
// the schedule tabulated once in LDS.  One round costs one barrier:
//   * every wavefront computes all M/2 plane rotations redundantly (lane l owns
//     pair l mod M/2) from the current matrix, so no cross-wave exchange of the
//     rotations is needed; a thread fetches the two it needs by lane shuffle;
//   * thread (a, b) rewrites the 2x2 block (pair a) x (pair b) as J_a^T B J_b,
//     reading the current copy of the matrix and writing the other copy
//     (double buffering removes the read/write hazard inside a round);
//   * the same thread applies J_a to two rows of the eigenvector matrix.
// Reciprocal square roots come from the hardware estimate refined by Newton steps
// to full double precision; the matrix is pre-scaled by a power of two so that
// squares cannot overflow or vanish.
#include "qn_internal.h"
#include "qn_project.h"

namespace qn {

constexpr int kEigMaxSweeps = 30;
// A power of two (the block reductions are trees).  Above M = 32 a thread takes
// several of the (M/2)^2 blocks of a round; measured best: 512 threads at M = 48
// (359 us against 384 with 1024), 256 at M = 64 (709 us against 832 with 1024).
// Up to M = 8 one wavefront holds every block (25 us against 30 with four).
// M = 16: the 64 blocks of a round are one wavefront's worth (50 us against 54)
#ifndef QN_EIG_THREADS_16
#define QN_EIG_THREADS_16 64
#endif
#ifndef QN_EIG_THREADS_24
#define QN_EIG_THREADS_24 256
#endif
#ifndef QN_EIG_THREADS_32
#define QN_EIG_THREADS_32 256
#endif
template <int M> constexpr int eig_threads()
{
    return M <= 8 ? 64
                  : (M == 16 ? QN_EIG_THREADS_16
                             : (M == 24 ? QN_EIG_THREADS_24
                                        : (M == 32 ? QN_EIG_THREADS_32 : (M == 48 ? 512 : 256))));
}
// dynamic LDS: two copies of the matrix and the eigenvectors, leading dimension M + 1
template <int M> constexpr int eig_lds_bytes() { return 3 * M * (M + 1) * static_cast<int>(sizeof(double)); }

// Workgroup reductions in a fixed order: butterfly inside each wavefront, then the
// wave results in wave order.  Two barriers (the second frees scratch for reuse).
template <int THREADS>
__device__ __forceinline__ double block_sum(double v, double *scratch)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_xor(v, off);
    if ((threadIdx.x & 63) == 0)
        scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int wv = 0; wv < THREADS / 64; ++wv)
        r += scratch[wv];
    __syncthreads();
    return r;
}

template <int THREADS>
__device__ __forceinline__ double block_max(double v, double *scratch)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        v = fmax(v, __shfl_xor(v, off));
    if ((threadIdx.x & 63) == 0)
        scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = scratch[0];
#pragma unroll
    for (int wv = 1; wv < THREADS / 64; ++wv)
        r = fmax(r, scratch[wv]);
    __syncthreads();
    return r;
}

// 1/sqrt(x) to double precision: hardware estimate + Newton steps.
__device__ __forceinline__ double fast_rsqrt(double x)
{
    double r = __builtin_amdgcn_rsq(x);
    // the estimate is good to about 5e-8 (measured): r <- r + r*(1 - x r^2)/2, twice
    double e = fma(-x * r, r, 1.0);
    r = fma(0.5 * r, e, r);
    e = fma(-x * r, r, 1.0);
    r = fma(0.5 * r, e, r);
    return r;
}

// Plane rotation J = [[c, s], [-s, c]] that annihilates the (p, q) entry of a
// symmetric matrix: theta with tan(2 theta) = 2 apq / (aqq - app), |theta| <= pi/4
// (t = tan(theta) is the smaller root of t^2 + 2 zeta t - 1, zeta = (aqq - app) /
// (2 apq)).  From the half-angle formulas, with hyp = sqrt((aqq - app)^2 + 4 apq^2):
//     cos(2 theta) = |aqq - app| / hyp,   c = sqrt(X),  X = (1 + cos(2 theta)) / 2,
//     s = sgn(aqq - app) apq / (hyp c).
// Two reciprocal square roots (of hyp^2 and of X, which lies in [1/2, 1]) and no
// division: the shortest dependent chain found for the critical path of a round.
__device__ __forceinline__ void rotation(double app, double aqq, double apq,
                                         double &c, double &s)
{
    // Branch-free: a vanishing pair (apq = 0 with app = aqq, or both far below the
    // scaled matrix norm) takes the identity by selection.  apq = 0 alone gives
    // X = 1, c = 1, s = 0 through the formulas.
    const double delta = aqq - app, twice = 2.0 * apq;
    const double h2 = fma(delta, delta, twice * twice);
    const bool ok = h2 > 1e-290;
    const double r = fast_rsqrt(ok ? h2 : 1.0);                  // 1 / hyp
    const double X = fma(fabs(delta), 0.5 * r, 0.5);
    const double rc = fast_rsqrt(X);                             // 1 / c
    c = ok ? X * rc : 1.0;
    s = ok ? copysign(1.0, delta) * apq * r * rc : 0.0;
}

// Input: C and w in memory, or (C == nullptr) the raw accumulators of the Gram
// pass, from which the kernel forms C and w itself (qn_project.h), saving the
// launch of gram_project inside the fused entry points.
template <int M>
__global__ __launch_bounds__(eig_threads<M>()) void eig_select(
    const double *__restrict__ C, const double *__restrict__ w, int m,
    double lambda, double *__restrict__ sigma_out, double *__restrict__ V_out,
    float *__restrict__ c_out, int *__restrict__ j_out,
    const double *__restrict__ mraw, int entries, int z_mode, int pack,
    double *__restrict__ c64_out)
{
    constexpr int NP = M / 2;          // pairs per round
    constexpr int ROUNDS = M - 1;
    constexpr int LD = M + 1;          // padded leading dimension in LDS
    constexpr int kEigThreads = eig_threads<M>();
    extern __shared__ __attribute__((aligned(16))) double eig_lds[];
    double (*A)[M][LD] = reinterpret_cast<double (*)[M][LD]>(eig_lds);   // A[2][M][LD]
    double (*V)[LD] = reinterpret_cast<double (*)[LD]>(eig_lds + 2 * M * LD);
    // V[k][r]: component r of column k
    __shared__ double scratch[kEigThreads];
    __shared__ unsigned char sp[ROUNDS][NP], sq[ROUNDS][NP];
    __shared__ double wv[M], sig[M], coef[M], cvec[M];
    __shared__ int perm[M];
    __shared__ int bad, jsel;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    if (tid == 0)
        bad = 0;
    __syncthreads();

    // symmetric part, zero padding, V = I, non-finite scan, schedule
    if (C == nullptr) {
        // from the raw accumulators: C lands in A[0], w in wv; the second copy of
        // the matrix is free to serve as the projection's work space
        __shared__ ProjectScratch sc;
        __shared__ double red[gram_entries(M)];
        project_raw<kEigThreads>(
            mraw, entries, m, z_mode, pack, &A[1][0][0], LD, red, sc,
            [&](int k, int l, double v) { A[0][k][l] = v; },
            [&](int k, double v) { wv[k] = v; });
    }
    double amax = 0.0;
    for (int e = tid; e < M * M; e += kEigThreads) {
        const int k = e / M, l = e % M;
        double v = 0.0;
        if (k < m && l < m) {
            v = C != nullptr ? 0.5 * (C[l * m + k] + C[k * m + l]) : A[0][k][l];
            if (!isfinite(v))
                bad = 1;
            amax = fmax(amax, fabs(v));
        }
        A[0][k][l] = v;
        V[k][l] = (k == l) ? 1.0 : 0.0;
    }
    if (tid < m) {
        if (C != nullptr)
            wv[tid] = w[tid];
        if (!isfinite(wv[tid]))
            bad = 1;
    }
    for (int e = tid; e < ROUNDS * NP; e += kEigThreads) {
        const int round = e / NP, i = e % NP;
        int p, q;
        if (i == 0) {
            p = round;
            q = M - 1;
        } else {
            p = (round + i) % (M - 1);
            q = (round - i + (M - 1)) % (M - 1);
        }
        sp[round][i] = static_cast<unsigned char>(p < q ? p : q);
        sq[round][i] = static_cast<unsigned char>(p < q ? q : p);
    }
    __syncthreads();

    if (bad) {   // uniform: read after the barrier
        const double qnan = __longlong_as_double(0x7ff8000000000000LL);
        if (tid < m) {
            c_out[tid] = 0.0f;
            if (c64_out)
                c64_out[tid] = 0.0;
            if (sigma_out)
                sigma_out[tid] = qnan;
        }
        if (V_out)
            for (int e = tid; e < m * m; e += kEigThreads)
                V_out[e] = qnan;
        if (tid == 0)
            *j_out = -1;
        return;
    }

    // scale by a power of two so that the largest entry lies in [1, 2)
    amax = block_max<kEigThreads>(amax, scratch);
    int expo = 0;
    if (amax > 0.0)
        (void)frexp(amax, &expo);
    const double scale = ldexp(1.0, 1 - expo), unscale = ldexp(1.0, expo - 1);
    double tot = 0.0;
    for (int e = tid; e < M * M; e += kEigThreads) {
        const double v = A[0][e / M][e % M] * scale;
        A[0][e / M][e % M] = v;
        tot += v * v;
    }
    const double tol2 = 1e-28 * block_sum<kEigThreads>(tot, scratch);

    int cur = 0;
    // the NP x NP blocks (pair a) x (pair b) are dealt out BPT per thread
    constexpr int BPT = (NP * NP + kEigThreads - 1) / kEigThreads;
    // The pairing is the same in every sweep and does not depend on the data, so
    // the indices of the next round are read from the table while the current
    // round is still being worked on (one LDS round trip less after each barrier).
    // Measured: 5-8 % faster at M = 8 and 32, slower where a thread holds several
    // blocks or M/2 is not a power of two (M = 24, 48, 64), which read in place.
    constexpr bool PREFETCH = BPT == 1 && (NP & (NP - 1)) == 0;
    // One block per thread: its operands are fetched before the rotation arithmetic
    // (measured 4-9 % faster at M = 8 .. 32; with several blocks per thread, M = 48
    // and 64, the extra live registers and LDS queueing cost more than they save).
    constexpr bool HOIST = BPT == 1;
    const int pr = lane % NP;        // every wavefront: lane l computes the rotation of pair l mod NP
    // Row offsets (index * LD) rather than indices are carried from round to round:
    // the multiplications then sit in the prefetch, off the critical path.
    double *const Ab = &A[0][0][0];
    double *const Vb = &V[0][0];
    int rp = sp[0][pr], rq = sq[0][pr];
    int rpo = rp * LD, rqo = rq * LD;
    int p1o[BPT], q1o[BPT], p2[BPT], q2[BPT];
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
        const int blk = tid + i * kEigThreads;
        const int pa = (blk / NP) % NP, pb = blk % NP;
        p1o[i] = sp[0][pa] * LD; q1o[i] = sq[0][pa] * LD;
        p2[i] = sp[0][pb]; q2[i] = sq[0][pb];
    }
    for (int sweep = 0; sweep < kEigMaxSweeps; ++sweep) {
        double off = 0.0;
        for (int e = tid; e < M * M; e += kEigThreads) {
            const int k = e / M, l = e % M;
            if (k != l)
                off += A[cur][k][l] * A[cur][k][l];
        }
        if (block_sum<kEigThreads>(off, scratch) <= tol2)
            break;

        for (int round = 0; round < ROUNDS; ++round) {
            const double *const Ac = Ab + cur * (M * LD);
            double *const An = Ab + (cur ^ 1) * (M * LD);
            if constexpr (!PREFETCH) {       // the indices of this round, in place
                rp = sp[round][pr]; rq = sq[round][pr];
                rpo = rp * LD; rqo = rq * LD;
#pragma unroll
                for (int i = 0; i < BPT; ++i) {
                    const int blk = tid + i * kEigThreads;
                    const int pa = (blk / NP) % NP, pb = blk % NP;
                    p1o[i] = sp[round][pa] * LD; q1o[i] = sq[round][pa] * LD;
                    p2[i] = sp[round][pb]; q2[i] = sq[round][pb];
                }
            }
            // The three entries of this lane's pair first, then (HOIST) the operands
            // of this thread's block, which do not depend on the rotations: their
            // trip to LDS overlaps the rotation arithmetic.  (Left to itself the
            // compiler reads the diagonal only after testing the off-diagonal entry,
            // and the block operands only after the rotation: two more LDS round
            // trips on the critical path of every round.)
            double app = Ac[rpo + rp], aqq = Ac[rqo + rq], apq = Ac[rpo + rq];
            asm volatile("" ::: "memory");      // these three are issued first
            double b00[BPT], b01[BPT], b10[BPT], b11[BPT], vp0[BPT], vq0[BPT], vp1[BPT], vq1[BPT];
            auto load_block = [&](int i) {
                const int pb = (tid + i * kEigThreads) % NP;
                // the indices are in range also for the idle tail (blk >= NP * NP)
                b00[i] = Ac[p1o[i] + p2[i]]; b01[i] = Ac[p1o[i] + q2[i]];
                b10[i] = Ac[q1o[i] + p2[i]]; b11[i] = Ac[q1o[i] + q2[i]];
                // V <- V J_a on rows 2*pb, 2*pb + 1
                vp0[i] = Vb[p1o[i] + 2 * pb]; vq0[i] = Vb[q1o[i] + 2 * pb];
                vp1[i] = Vb[p1o[i] + 2 * pb + 1]; vq1[i] = Vb[q1o[i] + 2 * pb + 1];
            };
            if constexpr (HOIST)
                load_block(0);
            // PREFETCH: the indices of round + 1
            [[maybe_unused]] int rp_n = 0, rq_n = 0, p1_n[BPT], q1_n[BPT], p2_n[BPT], q2_n[BPT];
            if constexpr (PREFETCH) {
                const int nr = round + 1 < ROUNDS ? round + 1 : 0;
                rp_n = sp[nr][pr]; rq_n = sq[nr][pr];
#pragma unroll
                for (int i = 0; i < BPT; ++i) {
                    const int blk = tid + i * kEigThreads;
                    const int pa = (blk / NP) % NP, pb = blk % NP;
                    p1_n[i] = sp[nr][pa]; q1_n[i] = sq[nr][pa];
                    p2_n[i] = sp[nr][pb]; q2_n[i] = sq[nr][pb];
                }
            }
            asm volatile("" ::: "memory");      // the loads above stay above
            asm volatile("" : "+v"(app), "+v"(aqq), "+v"(apq));
            double rc, rs;
            rotation(app, aqq, apq, rc, rs);
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                const int blk = tid + i * kEigThreads;
                const int pa = blk / NP, pb = blk % NP;      // this block's pair indices
                // pa % NP < NP also for the idle tail, so the shuffles stay in range
                const double c1 = __shfl(rc, pa % NP), s1 = __shfl(rs, pa % NP);
                const double c2 = __shfl(rc, pb), s2 = __shfl(rs, pb);
                if constexpr (!HOIST)
                    load_block(i);
                if (blk < NP * NP) {
                    // B <- J_a^T B J_b
                    const double t00 = c1 * b00[i] - s1 * b10[i], t01 = c1 * b01[i] - s1 * b11[i];
                    const double t10 = s1 * b00[i] + c1 * b10[i], t11 = s1 * b01[i] + c1 * b11[i];
                    double n00 = c2 * t00 - s2 * t01, n01 = s2 * t00 + c2 * t01;
                    double n10 = c2 * t10 - s2 * t11, n11 = s2 * t10 + c2 * t11;
                    if (pa == pb) {   // the annihilated pair: exactly diagonal
                        n01 = 0.0;
                        n10 = 0.0;
                    }
                    An[p1o[i] + p2[i]] = n00;
                    An[p1o[i] + q2[i]] = n01;
                    An[q1o[i] + p2[i]] = n10;
                    An[q1o[i] + q2[i]] = n11;
                    Vb[p1o[i] + 2 * pb] = c1 * vp0[i] - s1 * vq0[i];
                    Vb[q1o[i] + 2 * pb] = s1 * vp0[i] + c1 * vq0[i];
                    Vb[p1o[i] + 2 * pb + 1] = c1 * vp1[i] - s1 * vq1[i];
                    Vb[q1o[i] + 2 * pb + 1] = s1 * vp1[i] + c1 * vq1[i];
                }
            }
            if constexpr (PREFETCH) {
                rp = rp_n; rq = rq_n;
                rpo = rp * LD; rqo = rq * LD;
#pragma unroll
                for (int i = 0; i < BPT; ++i) {
                    p1o[i] = p1_n[i] * LD; q1o[i] = q1_n[i] * LD;
                    p2[i] = p2_n[i]; q2[i] = q2_n[i];
                }
            }
            __syncthreads();
            cur ^= 1;
        }
    }

    // sort descending by counting; sigma = sqrt(max(mu, 0)); padded indices
    // (>= m) are never coupled to the others and are left out
    if (tid < m) {
        const double mu = A[cur][tid][tid];
        int rank = 0;
        for (int l = 0; l < m; ++l) {
            const double ml = A[cur][l][l];
            rank += (ml > mu) || (ml == mu && l < tid);
        }
        perm[rank] = tid;
        sig[rank] = mu > 0.0 ? sqrt(mu * unscale) : 0.0;
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
        if (c64_out)
            c64_out[tid] = cvec[tid] - mean;
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
               hipStream_t stream, const RawGram *raw, double *c64)
{
    const double *mraw = raw ? raw->mraw : nullptr;
    const int entries = raw ? raw->entries : 0, z_mode = raw ? raw->z_mode : 0,
              pack = raw ? raw->pack : 1;
    if (raw) {
        C = nullptr;
        w = nullptr;
    }
    TraceScope ts(QN_K_EIG, stream);
    const double lam = static_cast<double>(lambda);
#define QN_EIG_LAUNCH(MM)                                                            \
    hipLaunchKernelGGL(eig_select<MM>, dim3(1), dim3(eig_threads<MM>()),             \
                       eig_lds_bytes<MM>(), stream, C, w, m, lam, sigma, V, c, j_out,   \
                       mraw, entries, z_mode, pack, c64)
    if (m <= 2) QN_EIG_LAUNCH(2);
    else if (m <= 4) QN_EIG_LAUNCH(4);
    else if (m <= 8) QN_EIG_LAUNCH(8);
    else if (m <= 16) QN_EIG_LAUNCH(16);
    else if (m <= 24) QN_EIG_LAUNCH(24);
    else if (m <= 32) QN_EIG_LAUNCH(32);
    else if (m <= 48) QN_EIG_LAUNCH(48);
    else QN_EIG_LAUNCH(64);
#undef QN_EIG_LAUNCH
    return check_launch();
}

// The M = 64 instance keeps 98 KiB of matrices in dynamic LDS: per-device opt-in.
int setup_eig_kernels()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(eig_select<64>),
                               hipFuncAttributeMaxDynamicSharedMemorySize,
                               eig_lds_bytes<64>()) == hipSuccess
               ? QN_OK
               : QN_ELAUNCH;
}

}  // namespace qn
