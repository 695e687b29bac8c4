// The m x m centring algebra that turns the raw, pivot-shifted accumulators of
// the streaming Gram pass into C = G^T G and w (Section 2: G's columns are the
// worker gradients minus their row mean).  Shared by gram_project (which writes
// C and w to memory) and by eig_select (which starts from the raw accumulators
// and keeps C in LDS), so both produce the same bits.
//
// With D = [ s | grad_1 - s | ... ], N = D^T D restricted to k, l >= 1,
// t_k = d_k^T s (or d_k^T z when the pass carried a vector z) and the projector
// P = I - 11^T/m:   C = P N P,   w = P (t + N 1 / m)   (w = P t for z).
#pragma once

#include "qn_internal.h"

namespace qn {

__host__ __device__ constexpr int tile_index(int ti, int tj) { return ti * (ti + 1) / 2 + tj; }

// Position of Q[k][l] (k >= l) in the raw accumulator layout: tile (k/16, l/16)
// of the lower triangle, and inside a tile element (i, j) sits in register i%4
// of lane 16*(i/4) + j.
__device__ __forceinline__ int raw_index(int k, int l)
{
    const int tile = tile_index(k >> 4, l >> 4);
    const int i = k & 15, j = l & 15;
    return (tile * 4 + (i & 3)) * 64 + (i >> 2) * 16 + j;
}

// Q[k][l], k >= l, from the reduced accumulators: the kReduceRows rows of the
// two-level reduction added in order and, when `pack` row blocks share the tile
// (m <= 16 / pack), the partial Gram matrices of those blocks added too.
__device__ __forceinline__ double raw_entry(const double *__restrict__ mraw, int entries,
                                            int pack, int k, int l)
{
    const int mp = 16 / pack;
    double q = 0.0;
    for (int b = 0; b < pack; ++b) {
        const int at = raw_index(b * mp + k, b * mp + l);
        double part = 0.0;
        for (int r = 0; r < kReduceRows; ++r)
            part += mraw[r * entries + at];
        q += part;
    }
    return q;
}

// What the projection needs besides the matrix N itself (LDS).
struct ProjectScratch {
    double rowsum[QN_MAX_M], u[QN_MAX_M];
    double total, umean;
};

// All THREADS threads of the block call this.  mraw: kReduceRows rows of
// `entries` accumulators.  pack > 1 (m <= 16 / pack): the raw tile holds `pack`
// diagonal blocks of 16 / pack rows and columns, partial results for disjoint
// row sets, which are added.  N: m rows of leading dimension ldn in LDS
// (scratch); red: `entries` doubles in LDS (scratch).  On return (after a
// barrier) put_C(k, l, value) has been called for every entry of C and
// put_w(k, value) for every entry of w, each by one thread.
template <int THREADS, typename PutC, typename PutW>
__device__ __forceinline__ void project_raw(const double *__restrict__ mraw, int entries,
                                            int m, int z_mode, int pack, double *N, int ldn,
                                            double *red, ProjectScratch &sc, PutC put_C,
                                            PutW put_w)
{
    const int tid = threadIdx.x;
    const int mp = 16 / pack;        // only used when pack > 1
    // The rows of the two-level reduction added in order, entry by entry, into
    // LDS: consecutive threads read consecutive addresses and every thread's
    // loads are independent, so this costs one trip to memory instead of one
    // per matrix entry.
    for (int at = tid; at < entries; at += THREADS) {
        double v[kReduceRows];
#pragma unroll
        for (int r = 0; r < kReduceRows; ++r)
            v[r] = mraw[r * entries + at];
        double q = 0.0;
#pragma unroll
        for (int r = 0; r < kReduceRows; ++r)
            q += v[r];
        red[at] = q;
    }
    __syncthreads();
    // Q[k][l], k >= l
    auto raw = [&](int k, int l) { return red[raw_index(k, l)]; };
    for (int e = tid; e < m * m; e += THREADS) {
        const int k = e / m, l = e % m;
        double q = 0.0;
        if (k >= 1 && l >= 1) {
            const int hi = k >= l ? k : l, lo = k >= l ? l : k;
            if (pack == 1) {
                q = raw(hi, lo);
            } else {
                for (int b = 0; b < pack; ++b)
                    q += raw(b * mp + hi, b * mp + lo);
            }
        }
        N[k * ldn + l] = q;
    }
    __syncthreads();
    if (tid < m) {
        double s = 0.0;
        for (int x = 0; x < m; ++x)
            s += N[tid * ldn + x];
        sc.rowsum[tid] = s;
        double t = 0.0;
        if (tid >= 1) {
            if (pack == 1) {
                t = raw(tid, 0);
            } else {
                for (int b = 0; b < pack; ++b)
                    t += raw(b * mp + tid, b * mp);
            }
        }
        sc.u[tid] = z_mode ? t : t + s / m;
    }
    __syncthreads();
    if (tid == 0) {
        double s = 0.0, su = 0.0;
        for (int x = 0; x < m; ++x) {
            s += sc.rowsum[x];
            su += sc.u[x];
        }
        sc.total = s;
        sc.umean = su / m;
    }
    __syncthreads();
    for (int e = tid; e < m * m; e += THREADS) {
        const int k = e / m, l = e % m;
        put_C(k, l,
              N[k * ldn + l] - (sc.rowsum[k] + sc.rowsum[l]) / m +
                  sc.total / (static_cast<double>(m) * m));
    }
    if (tid < m)
        put_w(tid, sc.u[tid] - sc.umean);
    __syncthreads();
}

}  // namespace qn
