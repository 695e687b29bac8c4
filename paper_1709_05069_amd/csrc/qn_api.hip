// C ABI of libqn (declared in include/qn.h): argument validation, the
// per-device workspace, the optional per-kernel event tracing, and the
// composition of the kernels into the server step of Section 2, eq. (2)-(4).
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "qn_internal.h"

namespace qn {

// ---------------------------------------------------------------- workspace --
constexpr int kMaxDevices = 64;
static Workspace g_ws[kMaxDevices];
static bool g_ws_ready[kMaxDevices];
static std::mutex g_ws_mutex;

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int get_workspace(Workspace **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return QN_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (!g_ws_ready[dev]) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return QN_ELAUNCH;
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return QN_EARCH;
        if (setup_gram_kernels() != QN_OK || setup_apply_kernels() != QN_OK ||
            setup_eig_kernels() != QN_OK)
            return QN_ELAUNCH;
        Workspace ws{};
        ws.cu_count = prop.multiProcessorCount;
        const size_t b_part = align_up(sizeof(double) * kGramMaxBlocks * kMaxEntries, 256);
        const size_t b_mraw = align_up(sizeof(double) * kReduceRows * kMaxEntries, 256);
        const size_t b_C = align_up(sizeof(double) * QN_MAX_M * QN_MAX_M, 256);
        const size_t b_w = align_up(sizeof(double) * QN_MAX_M, 256);
        const size_t b_c = align_up(sizeof(float) * QN_MAX_M, 256);
        ws.bytes = b_part + b_mraw + 3 * b_C + 4 * b_w + 3 * b_c;
        if (hipMalloc(&ws.base, ws.bytes) != hipSuccess) {
            (void)hipGetLastError();
            return QN_ENOMEM;
        }
        char *p = static_cast<char *>(ws.base);
        ws.partials = reinterpret_cast<double *>(p); p += b_part;
        ws.mraw = reinterpret_cast<double *>(p); p += b_mraw;
        ws.C = reinterpret_cast<double *>(p); p += b_C;
        ws.w = reinterpret_cast<double *>(p); p += b_w;
        ws.c = reinterpret_cast<float *>(p); p += b_c;
        ws.V = reinterpret_cast<double *>(p); p += b_C;
        ws.sigma = reinterpret_cast<double *>(p); p += b_w;
        ws.wz = reinterpret_cast<double *>(p); p += b_w;
        ws.cz = reinterpret_cast<float *>(p); p += b_c;
        ws.Ct = reinterpret_cast<double *>(p); p += b_C;
        ws.wt = reinterpret_cast<double *>(p); p += b_w;
        ws.tau_eff = reinterpret_cast<float *>(p); p += b_c;
        g_ws[dev] = ws;
        g_ws_ready[dev] = true;
    }
    *out = &g_ws[dev];
    return QN_OK;
}

// ------------------------------------------------------------------ tracing --
struct TraceState {
    bool enabled = false;
    int used = 0;
    std::vector<hipEvent_t> start, stop;
    std::vector<int> kernel;
};
static TraceState g_trace;

TraceScope::TraceScope(int kernel_id, hipStream_t s) : slot(-1), stream(s)
{
    if (g_trace.enabled && g_trace.used < static_cast<int>(g_trace.start.size())) {
        slot = g_trace.used++;
        g_trace.kernel[slot] = kernel_id;
        (void)hipEventRecord(g_trace.start[slot], stream);
    }
}

TraceScope::~TraceScope()
{
    if (slot >= 0)
        (void)hipEventRecord(g_trace.stop[slot], stream);
}

// --------------------------------------------------------------- validation --
static bool bad_common(const void *a, int dtype, int64_t n, int m, int64_t ld)
{
    return a == nullptr || (dtype != QN_F32 && dtype != QN_BF16 && dtype != QN_F16) || n < 1 ||
           m < 1 || m > QN_MAX_M || ld < n;
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
    Workspace *ws = nullptr;
    return get_workspace(&ws);
}

int qn_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    int cur = 0;
    if (hipGetDevice(&cur) != hipSuccess)
        return QN_ELAUNCH;
    int rc = QN_OK;
    for (int d = 0; d < kMaxDevices; ++d)
        if (g_ws_ready[d]) {
            if (hipSetDevice(d) != hipSuccess || hipFree(g_ws[d].base) != hipSuccess)
                rc = QN_ELAUNCH;
            g_ws_ready[d] = false;
        }
    (void)hipSetDevice(cur);
    return rc;
}

int qn_gram_ex(const void *grads, int dtype, int64_t n, int m, int64_t ld,
               double *C, double *w, qn_stream_t stream)
{
    if (bad_common(grads, dtype, n, m, ld) || !C || !w)
        return QN_EINVAL;
    Workspace *ws = nullptr;
    const int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    return launch_gram(grads, dtype, n, m, ld, ws, nullptr, C, w, static_cast<hipStream_t>(stream));
}

int qn_eig(const double *C, const double *w, int m, float lambda, double *sigma,
           double *V, float *c, int *j_out, qn_stream_t stream)
{
    if (!C || !w || !c || !j_out || m < 1 || m > QN_MAX_M ||
        !std::isfinite(lambda) || !(lambda > 0.0f))
        return QN_EINVAL;
    Workspace *ws = nullptr;   // arch check only
    const int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    return launch_eig(C, w, m, lambda, sigma, V, c, j_out, static_cast<hipStream_t>(stream));
}

int qn_apply_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                int m, int64_t ld, const float *c, float tau, float *theta_new,
                qn_stream_t stream)
{
    if (bad_common(thetas, dtype, n, m, ld) || !grads || !c || !theta_new ||
        !std::isfinite(tau))
        return QN_EINVAL;
    Workspace *ws = nullptr;
    const int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, c, nullptr, tau, nullptr, theta_new,
                        ws->cu_count, static_cast<hipStream_t>(stream));
}

int qn_update_ex(const void *thetas, const void *grads, int dtype, int64_t n,
                 int m, int64_t ld, float tau, float lambda, float *theta_new,
                 int *j_out, qn_stream_t stream)
{
    if (bad_common(thetas, dtype, n, m, ld) || !grads || !theta_new || !j_out ||
        !std::isfinite(tau) || !std::isfinite(lambda) || !(lambda > 0.0f))
        return QN_EINVAL;
    Workspace *ws = nullptr;
    int rc = get_workspace(&ws);
    if (rc != QN_OK)
        return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    RawGram raw;
    rc = launch_gram_raw(grads, dtype, n, m, ld, ws, nullptr, &raw, s);
    if (rc != QN_OK)
        return rc;
    rc = launch_eig(nullptr, nullptr, m, lambda, nullptr, nullptr, ws->c, j_out, s, &raw);
    if (rc != QN_OK)
        return rc;
    return launch_apply(thetas, grads, dtype, n, m, ld, ws->c, nullptr, tau, nullptr, theta_new,
                        ws->cu_count, s);
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
