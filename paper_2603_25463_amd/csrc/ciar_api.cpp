// C ABI of the library (include/ciar.h): argument validation, parameter resolution, launches.
// No allocation, no synchronisation; state: the thread-local error text, a launch counter (tags, see next_tag) and,
// for ciar_quantify_verify_static, the addresses of the built-in scratch buffer.
#include "../../include/ciar.h"
#include "ciar_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <chrono>
#include <mutex>

namespace {

thread_local char g_error[512] = "";

int fail(ciar_status code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return (int)code;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// z with P(|Z| <= z) = gamma for a standard normal Z, i.e. sqrt(2) * erfinv(gamma):
// Newton's method on erf(z / sqrt 2) - gamma from a closed-form starting point.
double two_sided_normal_quantile(double gamma)
{
    const double kPi = 3.14159265358979323846;
    // Winitzki's approximation of erfinv as the start
    const double a = 0.147, l = std::log(1.0 - gamma * gamma);
    const double t = 2.0 / (kPi * a) + 0.5 * l;
    double y = std::sqrt(std::sqrt(t * t - l / a) - t);          // ~ erfinv(gamma)
    for (int it = 0; it < 8; ++it) {
        const double f = std::erf(y) - gamma;
        const double d = 2.0 / std::sqrt(kPi) * std::exp(-y * y);
        y -= f / d;
    }
    return std::sqrt(2.0) * y;
}

struct Resolved {
    double a, b;       // e^{+r}, e^{-r} of the scalar radius r = min(kappa, radius_max)
    double kappa;      // radius scale
    int elt;           // bytes per logit
};

// Checks everything in `p` that does not depend on the tensors.  Returns CIAR_OK or fails.
int check_params(const ciar_params* p, Resolved* out)
{
    if (!p) return fail(CIAR_EINVAL, "params is NULL");
    if (p->struct_size != sizeof(ciar_params))
        return fail(CIAR_EINVAL, "params->struct_size is %u, expected %zu", p->struct_size, sizeof(ciar_params));
    if (p->reserved != 0) return fail(CIAR_EINVAL, "params->reserved must be 0");
    if (p->dtype != CIAR_F32 && p->dtype != CIAR_BF16)
        return fail(CIAR_EUNSUPPORTED, "params->dtype %d is neither CIAR_F32 nor CIAR_BF16", p->dtype);
    if (p->vocab < 1) return fail(CIAR_EINVAL, "params->vocab must be >= 1 (got %d)", p->vocab);
    if (p->vocab > ciar::max_vocab(p->dtype))
        return fail(CIAR_EUNSUPPORTED, "params->vocab %d exceeds the supported maximum %d for this dtype",
                    p->vocab, ciar::max_vocab(p->dtype));
    const int elt = p->dtype == CIAR_F32 ? 4 : 2;
    if (p->row_stride < p->vocab)
        return fail(CIAR_EINVAL, "params->row_stride %lld is smaller than vocab %d", (long long)p->row_stride,
                    p->vocab);
    if ((p->row_stride * elt) % 16 != 0)
        return fail(CIAR_EALIGN, "row_stride * element size = %lld bytes is not a multiple of 16",
                    (long long)(p->row_stride * elt));
    if (p->window < 1) return fail(CIAR_EINVAL, "params->window must be >= 1 (got %d)", p->window);
    if (!(p->radius_max >= 0.0f) || !(p->radius_max <= 16.0f))
        return fail(CIAR_EINVAL, "params->radius_max must be in [0, 16] (got %g)", (double)p->radius_max);
    if (!std::isfinite(p->tau)) return fail(CIAR_EINVAL, "params->tau must be finite");
    if (!(p->lower_cap > 0.0f) || !(p->lower_cap <= 1.0f) || !(p->upper_cap >= 1.0f) ||
        !std::isfinite(p->upper_cap))
        return fail(CIAR_EINVAL, "caps must satisfy 0 < lower_cap <= 1 <= upper_cap");
    double kappa;
    if (p->radius_scale >= 0.0f) {
        kappa = (double)p->radius_scale;
    } else {
        if (!(p->confidence > 0.0f) || !(p->confidence < 1.0f))
            return fail(CIAR_EINVAL, "params->confidence must be in (0, 1) when radius_scale < 0");
        kappa = two_sided_normal_quantile((double)p->confidence);
    }
    if (!std::isfinite(kappa)) return fail(CIAR_EINVAL, "params->radius_scale is not finite");
    const double r = kappa < (double)p->radius_max ? kappa : (double)p->radius_max;
    out->a = std::exp(r);
    out->b = std::exp(-r);
    out->kappa = kappa;
    out->elt = elt;
    return CIAR_OK;
}

int check_rows(const void* logits, const char* name)
{
    if (!logits) return fail(CIAR_EINVAL, "%s is NULL", name);
    if (!aligned16(logits)) return fail(CIAR_EALIGN, "%s is not 16-byte aligned", name);
    return CIAR_OK;
}

size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

// The width polynomial of a scalar radius (see RowArgs::wpoly).  With alpha = a - 1, beta = 1 - b:
//   G(x) = (1 - x) / ((1 + alpha x)(1 - beta x)) = 1 + x H(x),   H(x) = (beta - alpha - 1 + alpha beta x) / (same denominator)
// (H written so that nothing cancels).  P interpolates H at the four Chebyshev nodes of [0, rho]; rho is the
// largest interval, found by bisection, on which 1 + x P(x) stays within 2e-8 of G relative to G.
struct WidthPolyFit { double a, b; float c[4]; float x; };

double width_H(double alpha, double beta, double x)
{
    return (beta - alpha - 1.0 + alpha * beta * x) / ((1.0 + alpha * x) * (1.0 - beta * x));
}

// coefficients in s = x / rho and the largest relative error of 1 + x P(x) on (0, rho]
double width_fit(double alpha, double beta, double rho, double (&c)[4])
{
    static const double node[4] = {0.96193976625564337, 0.69134171618254492, 0.30865828381745508,
                                   0.03806023374435663};    // (1 + cos((2k+1) pi / 8)) / 2
    double f[4];
    for (int k = 0; k < 4; ++k) f[k] = width_H(alpha, beta, rho * node[k]);
    // Newton's divided differences, then the monomial coefficients by Horner expansion
    for (int lvl = 1; lvl < 4; ++lvl)
        for (int k = 3; k >= lvl; --k) f[k] = (f[k] - f[k - 1]) / (node[k] - node[k - lvl]);
    c[0] = f[3]; c[1] = c[2] = c[3] = 0.0;
    for (int k = 2; k >= 0; --k) {
        for (int j = 3; j >= 1; --j) c[j] = c[j - 1] - node[k] * c[j];
        c[0] = f[k] - node[k] * c[0];
    }
    double worst = 0.0;
    for (int i = 1; i <= 96; ++i) {
        const double sx = (double)i / 96.0, x = rho * sx;
        const double P = c[0] + sx * (c[1] + sx * (c[2] + sx * c[3]));
        const double G = 1.0 + x * width_H(alpha, beta, x);
        const double err = std::fabs(x * (P - width_H(alpha, beta, x))) / G;
        if (err > worst) worst = err;
    }
    return worst;
}

const WidthPolyFit& width_poly(double a, double b)
{
    static thread_local WidthPolyFit last = {-1.0, -1.0, {0.f, 0.f, 0.f, 0.f}, -1.f};
    if (last.a == a && last.b == b) return last;
    last.a = a; last.b = b; last.x = -1.f;
    last.c[0] = last.c[1] = last.c[2] = last.c[3] = 0.f;
    const double alpha = a - 1.0, beta = 1.0 - b;
    double lo = 0.0, hi = 0.25, c[4];
    for (int it = 0; it < 24; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (width_fit(alpha, beta, mid, c) <= 2e-8) lo = mid; else hi = mid;
    }
    if (lo >= 1e-6 && width_fit(alpha, beta, lo, c) <= 2e-8) {
        double s = 1.0;
        for (int j = 0; j < 4; ++j) { last.c[j] = (float)(c[j] * s); s /= lo; }   // back to powers of x
        last.x = (float)(lo * 0.999);
    }
    return last;
}

ciar::RowArgs base_args(const ciar_params* p, const Resolved& r, int64_t N)
{
    ciar::RowArgs a;
    std::memset(&a, 0, sizeof a);
    a.N = N;
    a.stride = p->row_stride;
    a.V = p->vocab;
    a.normalize = p->normalize ? 1 : 0;
    a.a = r.a;
    a.b = r.b;
    a.kappa = r.kappa;
    a.rmax = (double)p->radius_max;
    a.tau = (double)p->tau;
    a.cap_lo = (double)p->lower_cap;
    a.cap_hi = (double)p->upper_cap;
    // S_l <= b / (1 - (1-b) x_max) <= cap_lo  and  S_u >= a / (1 + (a-1) x_max) >= cap_hi  both hold when
    // x_max <= min((1 - b/cap_lo) / (1-b), (a/cap_hi - 1) / (a-1)); a hair below, to be safe against rounding.
    double xm = 0.0;
    if (r.a > 1.0) {
        const double x1 = (1.0 - r.b / a.cap_lo) / (1.0 - r.b), x2 = (r.a / a.cap_hi - 1.0) / (r.a - 1.0);
        xm = 0.999 * (x1 < x2 ? x1 : x2);
        if (!(xm > 0.0)) xm = 0.0;
    }
    a.capless_xmax = xm;
    a.precise_flat = 0;                                            // set by the callers that run the fp64 pass
    a.unit = 1;
    a.window = p->window;
    const WidthPolyFit& wf = width_poly(r.a, r.b);
    for (int j = 0; j < 4; ++j) a.wpoly[j] = wf.c[j];
    a.wpoly_x = wf.x;
    return a;
}

int hip_fail(hipError_t e, const char* what)
{
    return fail(CIAR_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// The launchers report hipGetLastError() after a launch.  HIP keeps that state per host thread and a successful call
// does not reset it, so an error left by an earlier, unrelated call of the thread is discarded before the first
// launch of an entry point: what is reported afterwards is this call's.
void discard_stale_hip_error() { (void)hipGetLastError(); }

// Workspace layout: [N] RowStats | [N] int32 row ids | [N] int32 arg-max tokens | 16 B (unused) | [N] uint8 accept bits
// (rounded up to 128 B) | 16 N bytes for the words of windows that span workgroups: window w at byte 16 K w, so that
// from K = 8 on every window has a 128-byte line of its own (the rows of many windows arrive at once, and atomic
// operations on one line are served one after another).
size_t stats_bytes(int64_t N) { return round_up((size_t)N * sizeof(ciar::RowStats), 16); }
size_t ids_bytes(int64_t N) { return round_up((size_t)N * 4, 16); }
size_t windows_offset(int64_t N) { return round_up(stats_bytes(N) + 2 * ids_bytes(N) + 16 + (size_t)N, 128); }

void carve(char* w, int64_t N, ciar::RowArgs* a, int32_t** row_ids, uint8_t** accept)
{
    a->stats = reinterpret_cast<ciar::RowStats*>(w);
    *row_ids = reinterpret_cast<int32_t*>(w + stats_bytes(N));
    a->reject_list = reinterpret_cast<int32_t*>(w + stats_bytes(N) + ids_bytes(N));
    *accept = reinterpret_cast<uint8_t*>(w + stats_bytes(N) + 2 * ids_bytes(N) + 16);
    a->win_words = reinterpret_cast<unsigned long long*>(w + windows_offset(N));
}

int check_workspace(int64_t N, const ciar_params* p, void* workspace, size_t workspace_bytes)
{
    if (N == 0) return CIAR_OK;
    const size_t need = ciar_workspace_bytes(N, p);
    if (!workspace) return fail(CIAR_EWORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (!aligned16(workspace)) return fail(CIAR_EALIGN, "workspace is not 16-byte aligned");
    if (workspace_bytes < need)
        return fail(CIAR_EWORKSPACE, "workspace has %zu bytes, %zu are needed", workspace_bytes, need);
    return CIAR_OK;
}

// Everything the three public passes share: validation, workspace carving, the two stages.
struct Call {
    const void* draft; const void* radius; const void* target; const int32_t* ids; const float* u_accept; const float* u_resample;
    int64_t N; const ciar_params* params;
    float* p_lo; float* p_mid; float* p_hi; float* omega; float* sigma; float* score; uint8_t* flags;
    uint8_t* accept; int32_t* row_id; int32_t* accept_len; int32_t* resampled_id;
    void* workspace; size_t workspace_bytes; hipStream_t stream;
    hipEvent_t ev_start = nullptr, ev_stop = nullptr;      // ciar_stream_rows_timed
};

bool wants_intervals(const Call& c)
{
    return c.p_lo || c.p_mid || c.p_hi || c.omega || c.sigma || c.score || c.flags;
}
bool wants_verify(const Call& c) { return c.accept || c.row_id || c.accept_len || c.resampled_id; }

// Validates what every stage needs and fills `a` (without the per-row output pointers).
int prepare(const Call& c, ciar::Mode mode, ciar::RowArgs* a)
{
    Resolved r;
    if (int rc = check_params(c.params, &r)) return rc;
    if (c.N < 0) return fail(CIAR_EINVAL, "N is negative");
    if (c.N > 0x7fffffffLL) return fail(CIAR_EUNSUPPORTED, "N exceeds 2^31 - 1 rows per call");
    if (int rc = check_rows(c.draft, "draft_logits")) return rc;
    if (mode != ciar::Mode::Quantify)
        if (int rc = check_rows(c.target, "target_logits")) return rc;
    if (c.radius) {
        if (mode == ciar::Mode::Verify) return fail(CIAR_EINVAL, "radius given but no interval output is computed");
        if (int rc = check_rows(c.radius, "radius")) return rc;
    }
    *a = base_args(c.params, r, c.N);
    a->draft = c.draft;
    a->radius = c.radius;
    a->target = c.target;
    return CIAR_OK;
}

// Validates a call's arguments, carves the workspace and fills every pointer the two stages use.
int fill(const Call& c, ciar::Mode mode, ciar::RowArgs* a)
{
    if (int rc = prepare(c, mode, a)) return rc;
    if (mode != ciar::Mode::Quantify) {
        if (!c.ids) return fail(CIAR_EINVAL, "draft_ids is NULL");
        if (!c.u_accept) return fail(CIAR_EINVAL, "u_accept is NULL");
        if (!c.u_resample) return fail(CIAR_EINVAL, "u_resample is NULL");
    }
    if (!wants_intervals(c) && !wants_verify(c)) return fail(CIAR_EINVAL, "every output pointer is NULL");
    if (int rc = check_workspace(c.N, c.params, c.workspace, c.workspace_bytes)) return rc;
    if (c.N == 0) return CIAR_OK;
    int32_t* ws_ids; uint8_t* ws_accept;
    carve(static_cast<char*>(c.workspace), c.N, a, &ws_ids, &ws_accept);
    a->ids = c.ids; a->u_accept = c.u_accept; a->u_resample = c.u_resample;
    a->p_lo = c.p_lo; a->p_mid = c.p_mid; a->p_hi = c.p_hi;
    a->omega = c.omega; a->sigma = c.sigma; a->score = c.score; a->flags = c.flags;
    a->accept = c.accept;
    a->row_id = c.row_id;
    // the window outputs are assembled from the per-row accept bits and draws
    if ((c.accept_len || c.resampled_id) && !a->accept) a->accept = ws_accept;
    if ((c.accept_len || c.resampled_id) && !a->row_id) a->row_id = ws_ids;
    if (a->row_id && !a->accept) a->accept = ws_accept;           // (resample_kernel finds its rows by their accept bits)
    a->window = c.params->window;
    a->accept_len = c.accept_len;
    a->resampled_id = c.resampled_id;
    return CIAR_OK;
}

// Tensor mode reports the arg-max token's interval with that token's own radius: without drafted ids the index
// comes from a kernel of its own, into a workspace array of N ints.
bool needs_argmax(const ciar::RowArgs& a) { return a.radius && !a.ids && (a.p_lo || a.p_hi); }

// Tags for the words the streaming kernel keeps in caller memory (see window_arrive in ciar_device.h): a different
// one for every launch of the process, starting from a value that varies from run to run.  (A captured graph replays
// a launch with its tag: the kernel hands every word back, with a zero tag, when a window is complete.)
uint32_t next_tag()
{
    static std::atomic<uint32_t> tag{(uint32_t)std::chrono::steady_clock::now().time_since_epoch().count() * 2654435761u};
    for (;;) {
        const uint32_t t = tag.fetch_add(1, std::memory_order_relaxed) + 1;
        if ((t & 0x7fffffffu) != 0) return t;                      // (a zero tag marks a word that has been handed back)
    }
}

// Stage 1: the streaming kernel, which also finishes its rows (and the fp64 pass over flat rows where the call needs it).
int run_stream(const Call& c, ciar::Mode mode)
{
    ciar::RowArgs a;
    if (int rc = fill(c, mode, &a)) return rc;
    if (c.N == 0) return CIAR_OK;
    discard_stale_hip_error();
    if (needs_argmax(a)) {
        const hipError_t e = ciar::launch_argmax(c.params->dtype, a, a.reject_list, c.stream);
        if (e != hipSuccess) return hip_fail(e, "arg-max kernel launch");
        a.ids = a.reject_list;
    }
    a.precise_flat = mode != ciar::Mode::Verify && ciar::needs_flat_pass(a) ? 1 : 0;
    a.tag = next_tag();
    hipError_t e = ciar::launch_stream(mode, c.params->dtype, a, true, c.stream, c.ev_start, c.ev_stop);
    if (e != hipSuccess) return hip_fail(e, "streaming kernel launch");
    if (a.precise_flat) {
        // flat rows of a call whose widths are not small: their interval sums again, in fp64
        const ciar::StreamPlan plan = ciar::plan_stream(mode, c.params->dtype, a);
        e = ciar::launch_flatrows(c.params->dtype, a, plan.can_finish, c.stream);
        if (e != hipSuccess) return hip_fail(e, "flat-row kernel launch");
    }
    return CIAR_OK;
}

// Stage 2: the window outputs, where the windows do not lie inside the streaming kernel's workgroups.
int run_finish(const Call& c, ciar::Mode mode)
{
    ciar::RowArgs a;
    if (int rc = fill(c, mode, &a)) return rc;
    if (c.N == 0) return CIAR_OK;
    if (needs_argmax(a)) a.ids = a.reject_list;                    // found by stage 1
    discard_stale_hip_error();
    const ciar::StreamPlan plan = ciar::plan_stream(mode, c.params->dtype, a);
    const hipError_t e = ciar::launch_finish(mode, c.params->dtype, a, plan, c.params->window, c.accept_len,
                                             c.resampled_id, c.stream);
    if (e != hipSuccess) return hip_fail(e, "finishing kernel launch");
    return CIAR_OK;
}

int run_both(const Call& c, ciar::Mode mode)
{
    if (int rc = run_stream(c, mode)) return rc;
    return run_finish(c, mode);
}

}  // namespace

// ---- the allocation-free variant of the fused call ------------------------------------------------------------
//
// The workspace of ciar_quantify_verify_static: one array per GPU the library runs on, held until the process ends.
// The name below is a host-side stand-in for the device array: host code never passes it anywhere but to
// hipGetSymbolAddress, and uses the address that call returns for the device that was current.
namespace {

constexpr int64_t kStaticRows = CIAR_STATIC_MAX_ROWS;
constexpr size_t static_round(size_t x, size_t m) { return (x + m - 1) / m * m; }
constexpr size_t kStaticBytes =
    static_round(static_round(static_round((size_t)kStaticRows * sizeof(ciar::RowStats), 16) +
                              2 * static_round((size_t)kStaticRows * 4, 16) + 16 + (size_t)kStaticRows, 128) +
                 16 * (size_t)kStaticRows, 256);      // = ciar_workspace_bytes(kStaticRows)

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// The address of `scratch` on the current device (asked once per device, with that device current).
int static_scratch(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(CIAR_EUNSUPPORTED, "device ordinal %d is outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p) return fail(CIAR_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CIAR_OK;
}

}  // namespace


extern "C" {

void ciar_params_default(ciar_params* p)
{
    if (!p) return;
    std::memset(p, 0, sizeof *p);
    p->struct_size = (uint32_t)sizeof(ciar_params);
    p->dtype = CIAR_F32;
    p->window = 8;
    p->confidence = 0.9f;
    p->radius_scale = -1.0f;
    p->radius_max = 10.0f;
    p->tau = 0.30f;
    p->lower_cap = 0.99f;
    p->upper_cap = 1.01f;
    p->normalize = 1;
}

int ciar_width_polynomial(const ciar_params* params, float* coef, float* x_max)
{
    if (!coef || !x_max) return fail(CIAR_EINVAL, "coef or x_max is NULL");
    Resolved r;
    if (int rc = check_params(params, &r)) return rc;
    const WidthPolyFit& wf = width_poly(r.a, r.b);
    for (int j = 0; j < 4; ++j) coef[j] = wf.c[j];
    *x_max = wf.x;
    return CIAR_OK;
}

size_t ciar_workspace_bytes(int64_t N, const ciar_params* /*params*/)
{
    if (N <= 0) return 0;
    return round_up(windows_offset(N) + 16 * (size_t)N, 256);
}

int ciar_quantify(const void* draft_logits, const void* radius, const int32_t* draft_ids, int64_t N,
                  const ciar_params* params, float* p_lo, float* p_mid, float* p_hi, float* omega, float* sigma,
                  float* score, uint8_t* flags, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const Call c{draft_logits, radius, nullptr, draft_ids, nullptr, nullptr, N, params, p_lo, p_mid, p_hi, omega, sigma,
                 score, flags, nullptr, nullptr, nullptr, nullptr, workspace, workspace_bytes,
                 static_cast<hipStream_t>(hip_stream)};
    return run_both(c, ciar::Mode::Quantify);
}

int ciar_verify(const void* draft_logits, const void* target_logits, const int32_t* draft_ids,
                const float* u_accept, const float* u_resample, int64_t N, const ciar_params* params,
                uint8_t* accept, int32_t* row_resample_id, int32_t* accept_len, int32_t* resampled_id,
                void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const Call c{draft_logits, nullptr, target_logits, draft_ids, u_accept, u_resample, N, params, nullptr, nullptr,
                 nullptr, nullptr, nullptr, nullptr, nullptr, accept, row_resample_id, accept_len, resampled_id,
                 workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream)};
    return run_both(c, ciar::Mode::Verify);
}

int ciar_quantify_verify(const void* draft_logits, const void* radius, const void* target_logits,
                         const int32_t* draft_ids, const float* u_accept, const float* u_resample, int64_t N,
                         const ciar_params* params, float* p_lo, float* p_mid, float* p_hi, float* omega,
                         float* sigma, float* score, uint8_t* flags, uint8_t* accept, int32_t* row_resample_id,
                         int32_t* accept_len, int32_t* resampled_id, void* workspace, size_t workspace_bytes,
                         void* hip_stream)
{
    const Call c{draft_logits, radius, target_logits, draft_ids, u_accept, u_resample, N, params, p_lo, p_mid, p_hi, omega,
                 sigma, score, flags, accept, row_resample_id, accept_len, resampled_id, workspace, workspace_bytes,
                 static_cast<hipStream_t>(hip_stream)};
    return run_both(c, ciar::Mode::Fused);
}

int ciar_stream_rows(const void* draft_logits, const void* radius, const void* target_logits,
                     const int32_t* draft_ids, const float* u_accept, const float* u_resample, int64_t N,
                     const ciar_params* params, float* p_lo, float* p_mid, float* p_hi, float* omega, float* sigma,
                     float* score, uint8_t* flags, uint8_t* accept, int32_t* row_resample_id, int32_t* accept_len,
                     int32_t* resampled_id, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const Call c{draft_logits, radius, target_logits, draft_ids, u_accept, u_resample, N, params, p_lo, p_mid, p_hi, omega,
                 sigma, score, flags, accept, row_resample_id, accept_len, resampled_id, workspace, workspace_bytes,
                 static_cast<hipStream_t>(hip_stream)};
    if (target_logits && !wants_verify(c)) return fail(CIAR_EINVAL, "target_logits given but no verify output");
    if (!target_logits && wants_verify(c)) return fail(CIAR_EINVAL, "verify outputs need target_logits");
    const ciar::Mode mode = !target_logits ? ciar::Mode::Quantify
                                           : (wants_intervals(c) ? ciar::Mode::Fused : ciar::Mode::Verify);
    return run_stream(c, mode);
}

int ciar_stream_rows_timed(const void* draft_logits, const void* radius, const void* target_logits,
                           const int32_t* draft_ids, const float* u_accept, const float* u_resample, int64_t N,
                           const ciar_params* params, float* p_lo, float* p_mid, float* p_hi, float* omega,
                           float* sigma, float* score, uint8_t* flags, uint8_t* accept, int32_t* row_resample_id,
                           int32_t* accept_len, int32_t* resampled_id, void* workspace, size_t workspace_bytes,
                           void* hip_stream, void* start_event, void* stop_event)
{
    if (!start_event || !stop_event) return fail(CIAR_EINVAL, "start_event or stop_event is NULL");
    Call c{draft_logits, radius, target_logits, draft_ids, u_accept, u_resample, N, params, p_lo, p_mid, p_hi, omega,
           sigma, score, flags, accept, row_resample_id, accept_len, resampled_id, workspace, workspace_bytes,
           static_cast<hipStream_t>(hip_stream)};
    c.ev_start = static_cast<hipEvent_t>(start_event);
    c.ev_stop = static_cast<hipEvent_t>(stop_event);
    if (target_logits && !wants_verify(c)) return fail(CIAR_EINVAL, "target_logits given but no verify output");
    if (!target_logits && wants_verify(c)) return fail(CIAR_EINVAL, "verify outputs need target_logits");
    const ciar::Mode mode = !target_logits ? ciar::Mode::Quantify
                                           : (wants_intervals(c) ? ciar::Mode::Fused : ciar::Mode::Verify);
    return run_stream(c, mode);
}

int ciar_finish_rows(const void* draft_logits, const void* radius, const void* target_logits,
                     const int32_t* draft_ids, const float* u_accept, const float* u_resample, int64_t N,
                     const ciar_params* params, float* p_lo, float* p_mid, float* p_hi, float* omega, float* sigma,
                     float* score, uint8_t* flags, uint8_t* accept, int32_t* row_resample_id, int32_t* accept_len,
                     int32_t* resampled_id, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const Call c{draft_logits, radius, target_logits, draft_ids, u_accept, u_resample, N, params, p_lo, p_mid, p_hi, omega,
                 sigma, score, flags, accept, row_resample_id, accept_len, resampled_id, workspace, workspace_bytes,
                 static_cast<hipStream_t>(hip_stream)};
    if (target_logits && !wants_verify(c)) return fail(CIAR_EINVAL, "target_logits given but no verify output");
    if (!target_logits && wants_verify(c)) return fail(CIAR_EINVAL, "verify outputs need target_logits");
    const ciar::Mode mode = !target_logits ? ciar::Mode::Quantify
                                           : (wants_intervals(c) ? ciar::Mode::Fused : ciar::Mode::Verify);
    return run_finish(c, mode);
}

int ciar_window_epilogue(const uint8_t* accept, const int32_t* row_resample_id, int64_t N,
                         const ciar_params* params, int32_t* accept_len, int32_t* resampled_id,
                         void* hip_stream)
{
    if (!params) return fail(CIAR_EINVAL, "params is NULL");
    if (params->struct_size != sizeof(ciar_params))
        return fail(CIAR_EINVAL, "params->struct_size is %u, expected %zu", params->struct_size,
                    sizeof(ciar_params));
    if (params->window < 1) return fail(CIAR_EINVAL, "params->window must be >= 1 (got %d)", params->window);
    if (N < 0) return fail(CIAR_EINVAL, "N is negative");
    if (!accept) return fail(CIAR_EINVAL, "accept is NULL");
    if (!accept_len && !resampled_id) return fail(CIAR_EINVAL, "every output pointer is NULL");
    if (resampled_id && !row_resample_id)
        return fail(CIAR_EINVAL, "row_resample_id is NULL but resampled_id is requested");
    if (N == 0) return CIAR_OK;
    discard_stale_hip_error();
    hipError_t e = ciar::launch_windows(accept, row_resample_id, N, params->window, accept_len, resampled_id,
                                        static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "window kernel launch");
    return CIAR_OK;
}

int ciar_dense_intervals(const void* draft_logits, const void* radius, int64_t N, const ciar_params* params,
                         float* p_lo, float* p_mid, float* p_hi, void* hip_stream)
{
    Resolved r;
    if (int rc = check_params(params, &r)) return rc;
    if (N < 0) return fail(CIAR_EINVAL, "N is negative");
    if (int rc = check_rows(draft_logits, "draft_logits")) return rc;
    if (!p_lo && !p_mid && !p_hi) return fail(CIAR_EINVAL, "every output pointer is NULL");
    if (N > 0x7fffffffLL) return fail(CIAR_EUNSUPPORTED, "N exceeds 2^31 - 1 rows per call");
    if (radius)
        if (int rc = check_rows(radius, "radius")) return rc;
    ciar::RowArgs a = base_args(params, r, N);
    a.draft = draft_logits;
    a.radius = radius;
    if (N == 0) return CIAR_OK;
    discard_stale_hip_error();
    hipError_t e = ciar::launch_dense(params->dtype, a, p_lo, p_mid, p_hi, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "dense kernel launch");
    return CIAR_OK;
}

int ciar_interdro_loss(const void* center_logits, const void* radius, const void* cloud_logits, int64_t N,
                       const ciar_params* params, float lambda_v, float lambda_p, float lambda_beta, float alpha,
                       float* row_terms, float* weights, float* losses, void* hip_stream)
{
    Resolved r;
    if (int rc = check_params(params, &r)) return rc;
    if (N < 0) return fail(CIAR_EINVAL, "N is negative");
    if (N > 0x7fffffffLL) return fail(CIAR_EUNSUPPORTED, "N exceeds 2^31 - 1 rows per call");
    if (int rc = check_rows(center_logits, "center_logits")) return rc;
    if (int rc = check_rows(cloud_logits, "cloud_logits")) return rc;
    if (radius)
        if (int rc = check_rows(radius, "radius")) return rc;
    if (!std::isfinite(lambda_v) || !std::isfinite(lambda_p) || !std::isfinite(lambda_beta) || !std::isfinite(alpha))
        return fail(CIAR_EINVAL, "lambda_v, lambda_p, lambda_beta and alpha must be finite");
    if (!row_terms) return fail(CIAR_EINVAL, "row_terms is NULL");
    if (N == 0) return CIAR_OK;
    ciar::RowArgs a = base_args(params, r, N);
    a.draft = center_logits;
    a.radius = radius;
    a.target = cloud_logits;
    discard_stale_hip_error();
    const hipError_t e = ciar::launch_dro(params->dtype, a, row_terms, lambda_v, lambda_p, lambda_beta, alpha, weights,
                                          losses, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "loss kernel launch");
    return CIAR_OK;
}

size_t ciar_multihead_workspace_bytes(int64_t N, int32_t heads, const ciar_params* /*params*/)
{
    if (N <= 0 || heads < 1) return 0;
    return round_up((size_t)heads * (stats_bytes(N) + ids_bytes(N) + round_up((size_t)N, 16)), 256);
}

int ciar_quantify_multihead(const void* draft_heads, const void* radius_heads, int32_t heads, int64_t head_stride,
                            const int32_t* draft_ids, int64_t N, const ciar_params* params, int32_t strategy,
                            float* p_lo, float* p_mid, float* p_hi, float* omega, float* sigma, float* score,
                            uint8_t* flags, uint8_t* head_flags, void* workspace, size_t workspace_bytes,
                            void* hip_stream)
{
    Resolved r;
    if (int rc = check_params(params, &r)) return rc;
    if (N < 0) return fail(CIAR_EINVAL, "N is negative");
    if (N > 0x7fffffffLL) return fail(CIAR_EUNSUPPORTED, "N exceeds 2^31 - 1 rows per call");
    if (heads < 1 || heads > ciar::max_heads())
        return fail(CIAR_EUNSUPPORTED, "heads must be in [1, %d] (got %d)", ciar::max_heads(), heads);
    if (strategy != CIAR_VOTING && strategy != CIAR_ENSEMBLE)
        return fail(CIAR_EINVAL, "strategy %d is neither CIAR_VOTING nor CIAR_ENSEMBLE", strategy);
    if (int rc = check_rows(draft_heads, "draft_heads")) return rc;
    if (radius_heads)
        if (int rc = check_rows(radius_heads, "radius_heads")) return rc;
    if (heads > 1) {
        if (head_stride < (N > 0 ? (N - 1) * params->row_stride + params->vocab : 0))
            return fail(CIAR_EINVAL, "head_stride %lld is smaller than one head's tensor", (long long)head_stride);
        if ((head_stride * r.elt) % 16 != 0)
            return fail(CIAR_EALIGN, "head_stride * element size is not a multiple of 16 bytes");
    }
    const bool any_float = p_lo || p_mid || p_hi || omega || sigma || score;
    if (!any_float && !flags && !(strategy == CIAR_VOTING && head_flags))
        return fail(CIAR_EINVAL, "every output pointer is NULL");
    if (N == 0) return CIAR_OK;
    const size_t need = ciar_multihead_workspace_bytes(N, heads, params);
    if (!workspace) return fail(CIAR_EWORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (!aligned16(workspace)) return fail(CIAR_EALIGN, "workspace is not 16-byte aligned");
    if (workspace_bytes < need)
        return fail(CIAR_EWORKSPACE, "workspace has %zu bytes, %zu are needed", workspace_bytes, need);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    discard_stale_hip_error();
    if (strategy == CIAR_ENSEMBLE) {
        // a few heads with a scalar radius whose rows fit the registers together: one sweep, every row read once
        ciar::RowArgs a = base_args(params, r, N);
        a.draft = draft_heads;
        a.radius = radius_heads;
        a.ids = draft_ids;
        a.p_lo = p_lo; a.p_mid = p_mid; a.p_hi = p_hi; a.omega = omega; a.sigma = sigma; a.score = score; a.flags = flags;
        if (ciar::ensemble_fused_fits(params->dtype, a, heads)) {
            const hipError_t e = ciar::launch_ensemble_fused(params->dtype, a, heads, head_stride, stream);
            if (e != hipSuccess) return hip_fail(e, "ensemble kernel launch");
            return CIAR_OK;
        }
    }
    char* w = static_cast<char*>(workspace);
    ciar::RowStats* stats = reinterpret_cast<ciar::RowStats*>(w);
    int32_t* ws_ids = reinterpret_cast<int32_t*>(w + (size_t)heads * stats_bytes(N));
    uint8_t* ws_flags = reinterpret_cast<uint8_t*>(w + (size_t)heads * (stats_bytes(N) + ids_bytes(N)));

    // one streaming pass over the rows of all heads ([heads, N] rows, head h at h * head_stride): every head's RowStats
    {
        const int64_t rows = (int64_t)heads * N;
        if (rows > 0x7fffffffLL) return fail(CIAR_EUNSUPPORTED, "heads * N exceeds 2^31 - 1 rows per call");
        ciar::RowArgs a = base_args(params, r, rows);
        if (heads > 1) { a.head_rows = N; a.head_stride = head_stride; }
        a.draft = draft_heads;
        a.radius = radius_heads;
        a.stats = stats;
        a.reject_list = ws_ids;                              // heads * N ints; a quantify-only pass builds no list
        if (strategy == CIAR_VOTING) {
            // every head is a quantifier of its own: the streaming kernel finishes its rows where it can;
            // the per-head outputs are [heads, N], which is the order of the rows
            a.ids = draft_ids;
            a.ids_period = heads > 1 ? N : 0;
            a.p_lo = p_lo; a.p_mid = p_mid; a.p_hi = p_hi;
            a.omega = omega; a.sigma = sigma; a.score = score;
            a.flags = head_flags ? head_flags : ws_flags;
            if (needs_argmax(a)) {
                const hipError_t e = ciar::launch_argmax(params->dtype, a, a.reject_list, stream);
                if (e != hipSuccess) return hip_fail(e, "arg-max kernel launch");
                a.ids = a.reject_list;
                a.ids_period = 0;
            }
            a.precise_flat = ciar::needs_flat_pass(a) ? 1 : 0;
            hipError_t e = ciar::launch_stream(ciar::Mode::Quantify, params->dtype, a, true, stream);
            if (e != hipSuccess) return hip_fail(e, "streaming kernel launch");
            const ciar::StreamPlan plan = ciar::plan_stream(ciar::Mode::Quantify, params->dtype, a);
            if (a.precise_flat) {
                e = ciar::launch_flatrows(params->dtype, a, plan.can_finish, stream);
                if (e != hipSuccess) return hip_fail(e, "flat-row kernel launch");
            }
        } else {
            // Ensemble: only every head's RowStats
            const hipError_t e = ciar::launch_stream(ciar::Mode::Quantify, params->dtype, a, false, stream);
            if (e != hipSuccess) return hip_fail(e, "streaming kernel launch");
        }
    }
    if (strategy == CIAR_VOTING) {
        if (flags) {
            const hipError_t e = ciar::launch_vote(head_flags ? head_flags : ws_flags, heads, N, flags, stream);
            if (e != hipSuccess) return hip_fail(e, "vote kernel launch");
        }
        return CIAR_OK;
    }
    ciar::RowArgs a = base_args(params, r, N);
    a.draft = draft_heads;
    a.radius = radius_heads;
    a.stats = stats;
    a.ids = draft_ids;
    a.p_lo = p_lo; a.p_mid = p_mid; a.p_hi = p_hi; a.omega = omega; a.sigma = sigma; a.score = score; a.flags = flags;
    const hipError_t e = ciar::launch_ensemble(params->dtype, a, heads, head_stride, stream);
    if (e != hipSuccess) return hip_fail(e, "ensemble kernel launch");
    return CIAR_OK;
}

namespace {
int read_rows(const void* draft_logits, const void* target_logits, int64_t N, const ciar_params* params,
              float* row_sum, void* hip_stream, hipEvent_t ev_start, hipEvent_t ev_stop);
}

int ciar_read_rows(const void* draft_logits, const void* target_logits, int64_t N, const ciar_params* params,
                   float* row_sum, void* hip_stream)
{
    return read_rows(draft_logits, target_logits, N, params, row_sum, hip_stream, nullptr, nullptr);
}

int ciar_read_rows_timed(const void* draft_logits, const void* target_logits, int64_t N, const ciar_params* params,
                         float* row_sum, void* hip_stream, void* start_event, void* stop_event)
{
    if (!start_event || !stop_event) return fail(CIAR_EINVAL, "start_event or stop_event is NULL");
    return read_rows(draft_logits, target_logits, N, params, row_sum, hip_stream, static_cast<hipEvent_t>(start_event),
                     static_cast<hipEvent_t>(stop_event));
}

namespace {
int read_rows(const void* draft_logits, const void* target_logits, int64_t N, const ciar_params* params,
              float* row_sum, void* hip_stream, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    Resolved r;
    if (int rc = check_params(params, &r)) return rc;
    if (N < 0) return fail(CIAR_EINVAL, "N is negative");
    if (N > 0x7fffffffLL) return fail(CIAR_EUNSUPPORTED, "N exceeds 2^31 - 1 rows per call");
    if (int rc = check_rows(draft_logits, "draft_logits")) return rc;
    if (target_logits)
        if (int rc = check_rows(target_logits, "target_logits")) return rc;
    if (!row_sum) return fail(CIAR_EINVAL, "row_sum is NULL");
    if (N == 0) return CIAR_OK;
    ciar::RowArgs a = base_args(params, r, N);
    a.draft = draft_logits;
    a.target = target_logits;
    discard_stale_hip_error();
    const hipError_t e = ciar::launch_read(params->dtype, a, row_sum, static_cast<hipStream_t>(hip_stream), ev_start,
                                           ev_stop);
    if (e != hipSuccess) return hip_fail(e, "read kernel launch");
    return CIAR_OK;
}
}  // namespace

namespace {
// Validation shared by the Interval Head entry points; fills everything of `h` but the two output tensors.
int head_args(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim, int64_t N,
              const ciar_params* params, ciar::HeadArgs* h)
{
    Resolved r;
    if (int rc = check_params(params, &r)) return rc;
    if (params->dtype != CIAR_F32)
        return fail(CIAR_EUNSUPPORTED, "the Interval Head produces fp32 logits: params->dtype must be CIAR_F32");
    if (N < 0) return fail(CIAR_EINVAL, "N is negative");
    if (N > 0x7fffffffLL) return fail(CIAR_EUNSUPPORTED, "N exceeds 2^31 - 1 rows per call");
    if (hidden_dim < ciar::kHeadTileDepth || hidden_dim % ciar::kHeadTileDepth != 0)
        return fail(CIAR_EUNSUPPORTED, "hidden_dim %d is not a positive multiple of %d", hidden_dim, ciar::kHeadTileDepth);
    if (params->vocab % ciar::kHeadTileCols != 0)
        return fail(CIAR_EUNSUPPORTED, "params->vocab %d is not a multiple of %d", params->vocab, ciar::kHeadTileCols);
    if (N > 0) {                                                   // an empty batch reads nothing
        if (int rc = check_rows(hidden, "hidden")) return rc;
        if (int rc = check_rows(weight, "weight")) return rc;
    }
    std::memset(h, 0, sizeof *h);
    h->hidden = static_cast<const uint16_t*>(hidden);
    h->weight = static_cast<const uint16_t*>(weight);
    h->bias = bias;
    h->N = N;
    h->stride = params->row_stride;
    h->D = hidden_dim;
    h->V = params->vocab;
    h->row_tiles = (int32_t)((N + ciar::kHeadTileRows - 1) / ciar::kHeadTileRows);
    return CIAR_OK;
}

size_t head_logit_bytes(int64_t N, const ciar_params* p) { return round_up((size_t)N * (size_t)p->row_stride * 4, 256); }

int head_logits(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim, int64_t N,
                const ciar_params* params, float* centre, float* radius, void* hip_stream, hipEvent_t ev_start,
                hipEvent_t ev_stop)
{
    ciar::HeadArgs h;
    if (int rc = head_args(hidden, weight, bias, hidden_dim, N, params, &h)) return rc;
    if (N == 0) return CIAR_OK;
    if (!centre || !radius) return fail(CIAR_EINVAL, "centre or radius is NULL");
    if (!aligned16(centre) || !aligned16(radius)) return fail(CIAR_EALIGN, "centre or radius is not 16-byte aligned");
    h.centre = centre;
    h.radius = radius;
    discard_stale_hip_error();
    const hipError_t e = ciar::launch_interhead(h, static_cast<hipStream_t>(hip_stream), ev_start, ev_stop);
    if (e != hipSuccess) return hip_fail(e, "Interval Head kernel launch");
    return CIAR_OK;
}
}  // namespace

size_t ciar_interhead_workspace_bytes(int64_t N, const ciar_params* params)
{
    if (N <= 0 || !params || params->row_stride <= 0) return 0;
    return 2 * head_logit_bytes(N, params) + ciar_workspace_bytes(N, params);
}

int ciar_interhead_logits(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim, int64_t N,
                          const ciar_params* params, float* centre, float* radius, void* hip_stream)
{
    return head_logits(hidden, weight, bias, hidden_dim, N, params, centre, radius, hip_stream, nullptr, nullptr);
}

int ciar_interhead_logits_timed(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim,
                                int64_t N, const ciar_params* params, float* centre, float* radius,
                                void* hip_stream, void* start_event, void* stop_event)
{
    if (!start_event || !stop_event) return fail(CIAR_EINVAL, "start_event or stop_event is NULL");
    return head_logits(hidden, weight, bias, hidden_dim, N, params, centre, radius, hip_stream,
                       static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event));
}

int ciar_interhead_quantify(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim,
                            const int32_t* draft_ids, int64_t N, const ciar_params* params, float* p_lo, float* p_mid,
                            float* p_hi, float* omega, float* sigma, float* score, uint8_t* flags, void* workspace,
                            size_t workspace_bytes, void* hip_stream)
{
    ciar::HeadArgs h;
    if (int rc = head_args(hidden, weight, bias, hidden_dim, N, params, &h)) return rc;
    if (N == 0) return CIAR_OK;                                    // an empty batch writes nothing
    if (!(p_lo || p_mid || p_hi || omega || sigma || score || flags))
        return fail(CIAR_EINVAL, "every output pointer is NULL");
    const size_t need = ciar_interhead_workspace_bytes(N, params);
    if (!workspace) return fail(CIAR_EWORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (!aligned16(workspace)) return fail(CIAR_EALIGN, "workspace is not 16-byte aligned");
    if (workspace_bytes < need)
        return fail(CIAR_EWORKSPACE, "workspace has %zu bytes, %zu are needed", workspace_bytes, need);
    char* w = static_cast<char*>(workspace);
    const size_t lb = head_logit_bytes(N, params);
    h.centre = reinterpret_cast<float*>(w);
    h.radius = reinterpret_cast<float*>(w + lb);
    discard_stale_hip_error();
    const hipError_t e = ciar::launch_interhead(h, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "Interval Head kernel launch");
    // the quantifier reads the logits the contraction has just written, on the same stream
    return ciar_quantify(h.centre, h.radius, draft_ids, N, params, p_lo, p_mid, p_hi, omega, sigma, score, flags,
                         w + 2 * lb, workspace_bytes - 2 * lb, hip_stream);
}


int ciar_quantify_verify_static(const void* draft_logits, const void* radius, const void* target_logits,
                                const int32_t* draft_ids, const float* u_accept, const float* u_resample, int64_t N,
                                const ciar_params* params, float* p_lo, float* p_mid, float* p_hi, float* omega,
                                float* sigma, float* score, uint8_t* flags, uint8_t* accept, int32_t* row_resample_id,
                                int32_t* accept_len, int32_t* resampled_id, void* hip_stream)
{
    if (N > kStaticRows)
        return fail(CIAR_EWORKSPACE, "N = %lld exceeds CIAR_STATIC_MAX_ROWS = %lld, the rows the built-in scratch "
                    "buffer holds: use ciar_quantify_verify with a workspace of the caller's", (long long)N,
                    (long long)kStaticRows);
    void* ws = nullptr;
    if (N > 0)
        if (int rc = static_scratch(&ws)) return rc;
    // Nothing in the buffer has to be cleared between calls: the window words carry the tag of the launch that wrote
    // them (and are handed back as zeros), everything else is written before it is read.
    const Call c{draft_logits, radius, target_logits, draft_ids, u_accept, u_resample, N, params, p_lo, p_mid, p_hi, omega,
                 sigma, score, flags, accept, row_resample_id, accept_len, resampled_id, ws, kStaticBytes,
                 static_cast<hipStream_t>(hip_stream)};
    return run_both(c, ciar::Mode::Fused);
}


const char* ciar_last_error(void) { return g_error; }

const char* ciar_version(void) { return "0.1.0"; }

}  // extern "C"
