// Internal declarations shared by the HIP translation units of libqn.
// Not part of the public ABI (that is include/qn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qn.h"

namespace qn {

// ---- fixed launch geometry -------------------------------------------------
// The Gram pass runs a fixed grid so that the summation tree depends only on
// (n, m, dtype, alignment) and the device's CU count.  Each block writes one
// partial; the partial holds the raw
// MFMA accumulator layout: kTileEntries values per 16x16 tile, 1, 3, 6 or 10
// tiles (the lower triangle of a 1x1 .. 4x4 tiling: m <= 16, 32, 48, 64).
#ifndef QN_GRAM_THREADS
#define QN_GRAM_THREADS 512                     // 8 wavefronts
#endif
constexpr int kGramThreads = QN_GRAM_THREADS;
constexpr int kGramWaves = kGramThreads / 64;
constexpr int kGramMaxBlocks = 1024;
constexpr int kTileEntries = 256;               // 16 x 16
constexpr int kMaxTiles = 10;                   // lower triangle of a 4x4 tiling (m <= 64)
constexpr int kMaxEntries = kTileEntries * kMaxTiles;
constexpr int kReduceRows = 8;                  // rows of the two-level partial reduction

// ---- per-device workspace ---------------------------------------------------
struct Workspace {
    double *partials;   // kGramMaxBlocks * kMaxEntries
    double *mraw;       // kReduceRows * kMaxEntries: reduced accumulators, raw tile layout
    double *C;          // QN_MAX_M * QN_MAX_M
    double *w;          // QN_MAX_M
    float *c;           // QN_MAX_M
    double *sigma;      // QN_MAX_M
    double *V;          // QN_MAX_M * QN_MAX_M
    double *wz;         // QN_MAX_M
    float *cz;          // QN_MAX_M
    double *Ct;         // QN_MAX_M * QN_MAX_M: Theta^T Theta for the secant bound
    double *wt;         // QN_MAX_M: by-product of that Gram pass (unused)
    float *tau_eff;     // 1: capped step size
    void *base;
    size_t bytes;
    int cu_count;
};

// Returns the current device's workspace (allocating it on first use).
int get_workspace(Workspace **out);

// ---- per-device kernel set-up (called once when a device's workspace is made) --
int setup_gram_kernels();
int setup_apply_kernels();
int setup_eig_kernels();

// ---- kernel launchers (each enqueues on `stream`, returns a qn_status) ------
// C = G^T G and, with z == nullptr, w = G^T g_bar; with z (n fp32 values) w = G^T z
int launch_gram(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                Workspace *ws, const float *z, double *C, double *w, hipStream_t stream);
// The raw, pivot-shifted accumulators of a Gram pass (kReduceRows rows of
// `entries` doubles in the workspace) and what is needed to decode them.
struct RawGram {
    const double *mraw;
    int entries;
    int z_mode;     // column 0 holds d_k^T z rather than d_k^T s
    int pack;       // row blocks packed into the single column set (m <= 8)
};
// stage 1 + reduce only; launch_gram adds the projection to C and w
int launch_gram_raw(const void *grads, int dtype, int64_t n, int m, int64_t ld,
                    Workspace *ws, const float *z, RawGram *raw, hipStream_t stream);
// raw != nullptr: C and w are formed inside the kernel from the raw accumulators
int launch_eig(const double *C, const double *w, int m, float lambda,
               double *sigma, double *V, float *c, int *j_out,
               hipStream_t stream, const RawGram *raw = nullptr);
// z == nullptr: theta_new = theta_bar - tau (g_bar + (Theta - G) c);
// z != nullptr: theta_new = z + (Theta - G) c  (tau unused);
// tau_dev != nullptr: tau is read from device memory instead of the argument
int launch_apply(const void *thetas, const void *grads, int dtype, int64_t n,
                 int m, int64_t ld, const float *c, const float *z, float tau,
                 const float *tau_dev, float *theta_new, int cu_count, hipStream_t stream);
// c = sum_{k < j} v_k (v_k^T w) / sigma_k^2, j read from device memory
int launch_coef(const double *sigma, const double *V, const int *j, const double *w,
                int m, float *c, hipStream_t stream);
// tau_out = min(tau, 1 / sigma_max) for the estimate named by mode (a qn_bound)
int launch_tau_bound(int mode, float tau, const double *sigma, const double *V,
                     const int *j, const double *Ct, int m, float *tau_out,
                     double *sigma_max_out, hipStream_t stream);

// ---- tracing ------------------------------------------------------------------
// RAII bracket: records a start/stop event pair around one kernel launch when
// tracing is enabled; otherwise does nothing.
struct TraceScope {
    TraceScope(int kernel_id, hipStream_t stream);
    ~TraceScope();
    int slot;
    hipStream_t stream;
};

inline int check_launch()
{
    return hipGetLastError() == hipSuccess ? QN_OK : QN_ELAUNCH;
}

}  // namespace qn
