// C ABI of libqn (declared in include/qn.h and include/qn_diag.h): argument
// validation, per-device set-up, workspaces, the optional per-kernel event
// tracing, and the composition of the kernels into the server step of Section 2,
// eq. (2)-(4).
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "qn_internal.h"

namespace qn {

// ---------------------------------------------------------- static scratch --
// Scratch memory of qn_update_noalloc: a device array inside the library's code
// object, so that the entry point needs neither hipMalloc nor a workspace argument.
// Every device the library runs on holds its own copy, at its own address, until
// the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: get_device() looks the address up once per device and the
// kernels are handed that pointer, never the name.  workspace_need() stays below
// this size for every problem on a device of up to 256 compute units.
constexpr size_t kStaticScratchBytes = 6u * 1024u * 1024u;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// ------------------------------------------------------------- device state --
constexpr int kMaxDevices = 64;
static Device g_dev[kMaxDevices];
static bool g_dev_ready[kMaxDevices];
static std::mutex g_dev_mutex;

int get_device(Device **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return QN_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    if (!g_dev_ready[dev]) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return QN_ELAUNCH;
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return QN_EARCH;
        if (setup_gram_kernels() != QN_OK || setup_apply_kernels() != QN_OK ||
            setup_eig_kernels() != QN_OK)
            return QN_ELAUNCH;
        Device d{};
        d.cu_count = prop.multiProcessorCount;
        // this device's copy of the static scratch array (the current device is `dev`)
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return QN_ELAUNCH;
        }
        d.static_scratch = ptr;
        g_dev[dev] = d;
        g_dev_ready[dev] = true;
    }
    *out = &g_dev[dev];
    return QN_OK;
}

int carve_workspace(void *base, size_t bytes, int64_t n, int m, int dtype, int cu_count,
                    Workspace *ws)
{
    if (base == nullptr || reinterpret_cast<uintptr_t>(base) % 256 != 0 ||
        bytes < workspace_need(n, m, dtype, cu_count))
        return QN_EWORKSPACE;
    const size_t entries = static_cast<size_t>(gram_entries(m));
    Workspace v{};
    v.cu_count = cu_count;
    v.max_partials = gram_max_partials(n, m, dtype, cu_count);
    char *p = static_cast<char *>(base);
    v.partials = reinterpret_cast<double *>(p);
    p += ws_align(sizeof(double) * static_cast<size_t>(v.max_partials) * entries);
    v.mraw = reinterpret_cast<double *>(p);
    p += ws_align(sizeof(double) * kReduceRows * entries);
    v.C = reinterpret_cast<double *>(p); p += kWsMatrixBytes;
    v.V = reinterpret_cast<double *>(p); p += kWsMatrixBytes;
    v.Ct = reinterpret_cast<double *>(p); p += kWsMatrixBytes;
    v.w = reinterpret_cast<double *>(p); p += kWsVectorBytes;
    v.sigma = reinterpret_cast<double *>(p); p += kWsVectorBytes;
    v.wz = reinterpret_cast<double *>(p); p += kWsVectorBytes;
    v.wt = reinterpret_cast<double *>(p); p += kWsVectorBytes;
    v.c = reinterpret_cast<float *>(p); p += kWsVectorBytes;
    v.cz = reinterpret_cast<float *>(p); p += kWsVectorBytes;
    v.tau_eff = reinterpret_cast<float *>(p); p += kWsVectorBytes;
    v.c64 = reinterpret_cast<double *>(p); p += kWsVectorBytes;
    v.cz64 = reinterpret_cast<double *>(p); p += kWsVectorBytes;
    *ws = v;
    return QN_OK;
}

// The largest workspace any problem needs on a device with this many units.
static size_t workspace_max(int cu_count)
{
    size_t best = 0;
    const int64_t big = static_cast<int64_t>(1) << 40;
    for (int m = 16; m <= QN_MAX_M; m += 16)
        for (int dt = QN_F32; dt <= QN_F16; ++dt) {
            const size_t b = workspace_need(big, m, dt, cu_count);
            best = b > best ? b : best;
        }
    return best;
}

int get_lib_workspace(int64_t n, int m, int dtype, Workspace *ws)
{
    Device *d = nullptr;
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    {
        std::lock_guard<std::mutex> lock(g_dev_mutex);
        if (d->lib_ws == nullptr) {
            const size_t bytes = workspace_max(d->cu_count);
            void *p = nullptr;
            if (hipMalloc(&p, bytes) != hipSuccess) {
                (void)hipGetLastError();
                return QN_ENOMEM;
            }
            d->lib_ws = p;
            d->lib_ws_bytes = bytes;
        }
    }
    return carve_workspace(d->lib_ws, d->lib_ws_bytes, n, m, dtype, d->cu_count, ws);
}

// A caller's buffer as the workspace of an (n, m, dtype) problem on the current device.
static int get_caller_workspace(void *base, size_t bytes, int64_t n, int m, int dtype,
                                Workspace *ws)
{
    Device *d = nullptr;
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    return carve_workspace(base, bytes, n, m, dtype, d->cu_count, ws);
}

// ------------------------------------------------------------------ tracing --
struct TraceState {
    bool enabled = false;
    int used = 0;
    std::vector<hipEvent_t> start, stop;
    std::vector<int> kernel;
};
static TraceState g_trace;
static std::mutex g_trace_mutex;

TraceScope::TraceScope(int kernel_id, hipStream_t s) : slot(-1), stream(s)
{
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    if (g_trace.enabled && g_trace.used < static_cast<int>(g_trace.start.size())) {
        slot = g_trace.used++;
        g_trace.kernel[slot] = kernel_id;
        (void)hipEventRecord(g_trace.start[slot], stream);
    }
}

TraceScope::~TraceScope()
{
    if (slot < 0)
        return;
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    if (g_trace.enabled && slot < static_cast<int>(g_trace.stop.size()))
        (void)hipEventRecord(g_trace.stop[slot], stream);
}

// ------------------------------------------------ the fused steps, any workspace --
int run_update(const void *thetas, const void *grads, int dtype, int64_t n, int m,
               int64_t ld, float tau, float lambda, float *theta_new, int *j_out,
               Workspace *ws, hipStream_t s)
{
    RawGram raw;
    int rc = launch_gram_raw(grads, dtype, n, m, ld, ws, nullptr, &raw, s);
    if (rc != QN_OK)
        return rc;
    // with fp32 storage the apply pass takes c in double (its sums run in fp64)
    double *c64 = dtype == QN_F32 ? ws->c64 : nullptr;
    rc = launch_eig(nullptr, nullptr, m, lambda, nullptr, nullptr, ws->c, j_out, s, &raw, c64);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, ws->c, nullptr, tau, nullptr, theta_new,
                        ws->cu_count, s, c64);
}

static bool bad_update_args(const void *thetas, const void *grads, int dtype, int64_t n,
                            int m, int64_t ld, float tau, float lambda,
                            const float *theta_new, const int *j_out)
{
    return bad_matrix_args(thetas, dtype, n, m, ld) || !grads || !theta_new || !j_out ||
           !std::isfinite(tau) || !std::isfinite(lambda) || !(lambda > 0.0f);
}

}  // namespace qn

using namespace qn;

extern "C" {

const char *qn_status_string(int status)
{
    switch (status) {
    case QN_OK: return "ok";
    case QN_EINVAL: return "invalid argument";
    case QN_ENOMEM: return "workspace allocation failed";
    case QN_ELAUNCH: return "HIP call or kernel launch failed";
    case QN_EARCH: return "device is not gfx950";
    case QN_EWORKSPACE: return "workspace missing, misaligned or too small";
    default: return "unknown status";
    }
}

const char *qn_kernel_name(int kernel_id)
{
    switch (kernel_id) {
    case QN_K_GRAM: return "gram_stage1";
    case QN_K_REDUCE: return "gram_reduce";
    case QN_K_PROJECT: return "gram_project";
    case QN_K_EIG: return "eig_select";
    case QN_K_APPLY: return "apply_kernel";
    case QN_K_COEF: return "coef";
    case QN_K_BOUND: return "tau_bound";
    default: return "unknown";
    }
}

int qn_init(void)
{
    Workspace ws;
    return get_lib_workspace(1, 1, QN_F32, &ws);
}

int qn_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_dev_mutex);
    int cur = 0;
    if (hipGetDevice(&cur) != hipSuccess)
        return QN_ELAUNCH;
    int rc = QN_OK;
    for (int d = 0; d < kMaxDevices; ++d)
        if (g_dev_ready[d] && g_dev[d].lib_ws != nullptr) {
            if (hipSetDevice(d) != hipSuccess || hipFree(g_dev[d].lib_ws) != hipSuccess)
                rc = QN_ELAUNCH;
            g_dev[d].lib_ws = nullptr;
            g_dev[d].lib_ws_bytes = 0;
        }
    (void)hipSetDevice(cur);
    return rc;
}

size_t qn_workspace_bytes(int64_t n, int m, int dtype)
{
    if (n < 1 || m < 1 || m > QN_MAX_M ||
        (dtype != QN_F32 && dtype != QN_BF16 && dtype != QN_F16))
        return 0;
    int cu = 256;
    Device *d = nullptr;
    if (get_device(&d) == QN_OK)
        cu = d->cu_count;
    return workspace_need(n, m, dtype, cu);
}

int qn_gram_ex(const void *grads, int dtype, int64_t n, int m, int64_t ld,
               double *C, double *w, qn_stream_t stream)
{
    if (bad_matrix_args(grads, dtype, n, m, ld) || !C || !w)
        return QN_EINVAL;
    Workspace ws;
    const int rc = get_lib_workspace(n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return launch_gram(grads, dtype, n, m, ld, &ws, nullptr, C, w, static_cast<hipStream_t>(stream));
}

int qn_gram_ws(const void *grads, int dtype, int64_t n, int m, int64_t ld, double *C,
               double *w, void *workspace, size_t workspace_bytes, qn_stream_t stream)
{
    if (bad_matrix_args(grads, dtype, n, m, ld) || !C || !w)
        return QN_EINVAL;
    Workspace ws;
    const int rc = get_caller_workspace(workspace, workspace_bytes, n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return launch_gram(grads, dtype, n, m, ld, &ws, nullptr, C, w, static_cast<hipStream_t>(stream));
}

int qn_diag_gram_ex(const void *grads, int dtype, const float *z, int64_t n, int m,
                    int64_t ld, int path, double *C, double *w, qn_stream_t stream)
{
    if (bad_matrix_args(grads, dtype, n, m, ld) || !C || !w ||
        (path != QN_GRAM_AUTO && path != QN_GRAM_STREAM && path != QN_GRAM_SMALL) ||
        (path == QN_GRAM_SMALL && n > (static_cast<int64_t>(1) << 22)))
        return QN_EINVAL;
    // a workspace that serves either kernel at any n: laid out for the largest grid
    Workspace ws;
    int rc = get_lib_workspace(static_cast<int64_t>(1) << 40, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return launch_gram(grads, dtype, n, m, ld, &ws, z, C, w, static_cast<hipStream_t>(stream), path);
}

int qn_eig(const double *C, const double *w, int m, float lambda, double *sigma,
           double *V, float *c, int *j_out, qn_stream_t stream)
{
    if (!C || !w || !c || !j_out || m < 1 || m > QN_MAX_M ||
        !std::isfinite(lambda) || !(lambda > 0.0f))
        return QN_EINVAL;
    Device *d = nullptr;   // architecture check and kernel set-up
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    return launch_eig(C, w, m, lambda, sigma, V, c, j_out, static_cast<hipStream_t>(stream));
}

int qn_apply_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                int m, int64_t ld, const float *c, float tau, float *theta_new,
                qn_stream_t stream)
{
    if (bad_matrix_args(thetas, dtype, n, m, ld) || !grads || !c || !theta_new ||
        !std::isfinite(tau))
        return QN_EINVAL;
    Device *d = nullptr;
    const int rc = get_device(&d);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, c, nullptr, tau, nullptr, theta_new,
                        d->cu_count, static_cast<hipStream_t>(stream));
}

int qn_update_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                 int m, int64_t ld, float tau, float lambda, float *theta_new,
                 int *j_out, qn_stream_t stream)
{
    if (bad_update_args(thetas, grads, dtype, n, m, ld, tau, lambda, theta_new, j_out))
        return QN_EINVAL;
    Workspace ws;
    const int rc = get_lib_workspace(n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return run_update(thetas, grads, dtype, n, m, ld, tau, lambda, theta_new, j_out, &ws,
                      static_cast<hipStream_t>(stream));
}

int qn_update_ws(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                 int64_t ld, float tau, float lambda, float *theta_new, int *j_out,
                 void *workspace, size_t workspace_bytes, qn_stream_t stream)
{
    if (bad_update_args(thetas, grads, dtype, n, m, ld, tau, lambda, theta_new, j_out))
        return QN_EINVAL;
    Workspace ws;
    const int rc = get_caller_workspace(workspace, workspace_bytes, n, m, dtype, &ws);
    if (rc != QN_OK)
        return rc;
    return run_update(thetas, grads, dtype, n, m, ld, tau, lambda, theta_new, j_out, &ws,
                      static_cast<hipStream_t>(stream));
}

int qn_update_noalloc(const void *thetas, const void *grads, int dtype, int64_t n, int m,
                      int64_t ld, float tau, float lambda, float *theta_new, int *j_out,
                      qn_stream_t stream)
{
    if (bad_update_args(thetas, grads, dtype, n, m, ld, tau, lambda, theta_new, j_out))
        return QN_EINVAL;
    Device *d = nullptr;
    int rc = get_device(&d);        // set-up only: no allocation
    if (rc != QN_OK)
        return rc;
    // the problem's scratch must fit the static array
    if (workspace_need(n, m, dtype, d->cu_count) > kStaticScratchBytes)
        return QN_EWORKSPACE;
    Workspace ws;
    rc = carve_workspace(d->static_scratch, kStaticScratchBytes, n, m, dtype, d->cu_count, &ws);
    if (rc != QN_OK)
        return rc;
    // Nothing in the scratch has to start at zero: every block of the Gram pass
    // writes its whole partial, the reduction reads exactly the partials of this
    // launch, and the eigen kernel writes c before the apply pass reads it.
    return run_update(thetas, grads, dtype, n, m, ld, tau, lambda, theta_new, j_out, &ws,
                      static_cast<hipStream_t>(stream));
}

int qn_update(const float *thetas, const float *grads, int64_t n, int m,
              float tau, float lambda, float *theta_new, int *j_out,
              qn_stream_t stream)
{
    return qn_update_ex(thetas, grads, QN_F32, n, m, n, tau, lambda, theta_new, j_out, stream);
}

int qn_update_bf16(const uint16_t *thetas, const uint16_t *grads, int64_t n,
                   int m, float tau, float lambda, float *theta_new, int *j_out,
                   qn_stream_t stream)
{
    return qn_update_ex(thetas, grads, QN_BF16, n, m, n, tau, lambda, theta_new, j_out, stream);
}

int qn_gram(const float *grads, int64_t n, int m, double *C, double *w,
            qn_stream_t stream)
{
    return qn_gram_ex(grads, QN_F32, n, m, n, C, w, stream);
}

int qn_gram_bf16(const uint16_t *grads, int64_t n, int m, double *C, double *w,
                 qn_stream_t stream)
{
    return qn_gram_ex(grads, QN_BF16, n, m, n, C, w, stream);
}

int qn_apply(const float *thetas, const float *grads, int64_t n, int m,
             const float *c, float tau, float *theta_new, qn_stream_t stream)
{
    return qn_apply_ex(thetas, grads, QN_F32, n, m, n, c, tau, theta_new, stream);
}

int qn_apply_bf16(const uint16_t *thetas, const uint16_t *grads, int64_t n,
                  int m, const float *c, float tau, float *theta_new,
                  qn_stream_t stream)
{
    return qn_apply_ex(thetas, grads, QN_BF16, n, m, n, c, tau, theta_new, stream);
}

int qn_trace_begin(int max_launches)
{
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    if (max_launches < 1 || g_trace.enabled)
        return QN_EINVAL;
    g_trace.start.resize(max_launches);
    g_trace.stop.resize(max_launches);
    g_trace.kernel.assign(max_launches, -1);
    for (int i = 0; i < max_launches; ++i)
        if (hipEventCreate(&g_trace.start[i]) != hipSuccess ||
            hipEventCreate(&g_trace.stop[i]) != hipSuccess)
            return QN_ELAUNCH;
    g_trace.used = 0;
    g_trace.enabled = true;
    return QN_OK;
}

int qn_trace_end(double *ms_sum, int *launches)
{
    std::lock_guard<std::mutex> lock(g_trace_mutex);
    if (!g_trace.enabled || !ms_sum || !launches)
        return QN_EINVAL;
    g_trace.enabled = false;
    for (int k = 0; k < QN_TRACE_KERNELS; ++k) {
        ms_sum[k] = 0.0;
        launches[k] = 0;
    }
    int rc = QN_OK;
    for (int i = 0; i < g_trace.used; ++i) {
        float ms = 0.0f;
        if (hipEventSynchronize(g_trace.stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_trace.start[i], g_trace.stop[i]) != hipSuccess) {
            rc = QN_ELAUNCH;
            continue;
        }
        const int k = g_trace.kernel[i];
        if (k >= 0 && k < QN_TRACE_KERNELS) {
            ms_sum[k] += ms;
            launches[k] += 1;
        }
    }
    for (size_t i = 0; i < g_trace.start.size(); ++i) {
        (void)hipEventDestroy(g_trace.start[i]);
        (void)hipEventDestroy(g_trace.stop[i]);
    }
    g_trace.start.clear();
    g_trace.stop.clear();
    g_trace.kernel.clear();
    g_trace.used = 0;
    return rc;
}

}  // extern "C"
