// Stand-ins for the kernel launchers and for the few HIP runtime calls of ciar_api.cpp, so that the C ABI's host
// code (validation, parameter resolution, workspace carving, the scratch-buffer lookup) links and runs on a machine
// without a GPU, under AddressSanitizer / UndefinedBehaviorSanitizer / ThreadSanitizer.  Every "device" pointer the
// driver passes is host memory of exactly the documented size, and each stub writes the full extent its kernel may
// write: a carve that leaves a region too small, or outside the workspace, is a heap overflow the sanitizer reports.
#include "../../paper_2603_25463_amd/csrc/ciar_internal.h"

#include <atomic>
#include <cstring>

namespace stubs {
std::atomic<int> launches{0};
std::atomic<int> stream_launches{0};
thread_local ciar::RowArgs last_args;
thread_local ciar::HeadArgs last_head;
}  // namespace stubs

namespace {
template <class T> void touch(T* p, size_t count)
{
    if (p && count) std::memset(static_cast<void*>(p), 0x5a, count * sizeof(T));
}
int64_t windows_of(const ciar::RowArgs& a) { return a.window > 0 ? (a.N + a.window - 1) / a.window : 0; }

void touch_row_outputs(const ciar::RowArgs& a)
{
    const size_t N = (size_t)a.N;
    touch(a.p_lo, N); touch(a.p_mid, N); touch(a.p_hi, N);
    touch(a.omega, N); touch(a.sigma, N); touch(a.score, N);
    touch(a.flags, N); touch(a.accept, N); touch(a.row_id, N);
    touch(a.stats, N);
}
}  // namespace

namespace ciar {

int max_vocab(int dtype) { return dtype == 0 ? 32768 : 65536; }
int max_heads() { return 8; }

StreamPlan plan_stream(Mode mode, int, const RowArgs& a, bool finish_rows)
{
    StreamPlan p{};
    p.grid = 1024; p.rows_per_wg = 4; p.can_finish = finish_rows; p.unit = 1;
    p.windows_inline = false;
    p.draws_inline = mode != Mode::Quantify && (a.N % 2 == 0);      // both finishing routes get exercised
    p.windows_counted = false;
    return p;
}

hipError_t launch_stream(Mode mode, int, const RowArgs& a, bool, hipStream_t, hipEvent_t, hipEvent_t)
{
    ++stubs::launches; ++stubs::stream_launches;
    stubs::last_args = a;
    touch_row_outputs(a);
    if (mode != Mode::Quantify) {
        touch(a.win_words, 2 * (size_t)a.N);                       // 16 bytes per row
        touch(a.accept_len, (size_t)windows_of(a)); touch(a.resampled_id, (size_t)windows_of(a));
    }
    return hipSuccess;
}
hipError_t launch_finish(Mode, int, const RowArgs& a, const StreamPlan&, int32_t K, int32_t* accept_len,
                         int32_t* resampled_id, hipStream_t)
{
    ++stubs::launches;
    const size_t W = (size_t)((a.N + K - 1) / K);
    touch(a.row_id, (size_t)a.N);
    touch(accept_len, W); touch(resampled_id, W);
    return hipSuccess;
}
hipError_t launch_flatrows(int, const RowArgs& a, bool, hipStream_t) { ++stubs::launches; touch_row_outputs(a); return hipSuccess; }
hipError_t launch_windows(const uint8_t*, const int32_t*, int64_t N, int32_t K, int32_t* accept_len, int32_t* resampled_id,
                          hipStream_t)
{
    ++stubs::launches;
    touch(accept_len, (size_t)((N + K - 1) / K)); touch(resampled_id, (size_t)((N + K - 1) / K));
    return hipSuccess;
}
hipError_t launch_dro(int, const RowArgs& a, float* terms, double, double, double, double, float* weights, float* losses,
                      hipStream_t)
{
    ++stubs::launches; stubs::last_args = a;
    touch(terms, 7 * (size_t)a.N); touch(weights, (size_t)a.N); touch(losses, 5);
    return hipSuccess;
}
hipError_t launch_ensemble(int, const RowArgs& a, int heads, int64_t, hipStream_t)
{
    ++stubs::launches; stubs::last_args = a;
    const size_t N = (size_t)a.N;
    touch(a.p_lo, N); touch(a.p_mid, N); touch(a.p_hi, N); touch(a.omega, N); touch(a.sigma, N); touch(a.score, N);
    touch(a.flags, N);
    touch(a.stats, (size_t)heads * N);
    return hipSuccess;
}
// (the one-sweep route is taken for a few heads with a scalar radius, as in the library)
bool ensemble_fused_fits(int, const RowArgs& a, int heads) { return !a.radius && heads <= 3 && a.V > 64 && a.V <= 16384; }
hipError_t launch_ensemble_fused(int, const RowArgs& a, int, int64_t, hipStream_t)
{
    ++stubs::launches; stubs::last_args = a;
    const size_t N = (size_t)a.N;
    touch(a.p_lo, N); touch(a.p_mid, N); touch(a.p_hi, N); touch(a.omega, N); touch(a.sigma, N); touch(a.score, N);
    touch(a.flags, N);
    return hipSuccess;
}
hipError_t launch_vote(const uint8_t* head_flags, int heads, int64_t N, uint8_t* flags, hipStream_t)
{
    ++stubs::launches;
    touch(const_cast<uint8_t*>(head_flags), (size_t)heads * (size_t)N); touch(flags, (size_t)N);
    return hipSuccess;
}
hipError_t launch_argmax(int, const RowArgs& a, int32_t* out, hipStream_t) { ++stubs::launches; touch(out, (size_t)a.N); return hipSuccess; }
hipError_t launch_dense(int, const RowArgs& a, float* lo, float* mid, float* hi, hipStream_t)
{
    ++stubs::launches;
    const size_t n = (size_t)a.N * (size_t)a.stride;
    touch(lo, n); touch(mid, n); touch(hi, n);
    return hipSuccess;
}
hipError_t launch_read(int, const RowArgs& a, float* row_sum, hipStream_t, hipEvent_t, hipEvent_t)
{
    ++stubs::launches; touch(row_sum, (size_t)a.N); return hipSuccess;
}
hipError_t launch_interhead(const HeadArgs& h, hipStream_t, hipEvent_t, hipEvent_t)
{
    ++stubs::launches; stubs::last_head = h;
    touch(h.centre, (size_t)h.N * (size_t)h.stride); touch(h.radius, (size_t)h.N * (size_t)h.stride);
    return hipSuccess;
}

}  // namespace ciar

// ---- the HIP runtime calls the C ABI makes itself ---------------------------------------------------------------
extern "C" {
hipError_t hipGetLastError(void) { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipGetDevice(int* dev) { *dev = 0; return hipSuccess; }
// (compiled as plain C++ the "device" array is a host array and HIP_SYMBOL(x) is x itself)
hipError_t hipGetSymbolAddress(void** p, const void* symbol) { *p = const_cast<void*>(symbol); return hipSuccess; }
}
