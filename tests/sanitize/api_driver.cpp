// Drives every host-side path of the C ABI against the stand-in launchers of api_stubs.cpp; built with sanitizers by
// tests/test_sanitizers.py.  Exit status 0 = every expectation held (the sanitizers abort the process otherwise).
#include "../../include/ciar.h"
#include "../../paper_2603_25463_amd/csrc/ciar_internal.h"

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

namespace stubs {
extern std::atomic<int> launches, stream_launches;
extern thread_local ciar::RowArgs last_args;
extern thread_local ciar::HeadArgs last_head;
}  // namespace stubs

static int g_failed = 0;
#define EXPECT(cond)                                                                                       \
    do {                                                                                                   \
        if (!(cond)) { std::fprintf(stderr, "%s:%d: EXPECT(%s) failed [%s]\n", __FILE__, __LINE__, #cond,  \
                                    ciar_last_error()); ++g_failed; }                                      \
    } while (0)

// 16-byte aligned host memory of exactly `bytes` bytes standing in for a device buffer
struct Buf {
    void* p = nullptr;
    // (an empty tensor still has an address: the C ABI rejects null tensors whatever N is)
    explicit Buf(size_t bytes) { if (posix_memalign(&p, 256, bytes ? bytes : 1)) std::abort(); }
    ~Buf() { std::free(p); }
    template <class T> T* as() const { return static_cast<T*>(p); }
};

static ciar_params params(int V, int dtype, int K)
{
    ciar_params p;
    ciar_params_default(&p);
    p.vocab = V; p.dtype = dtype; p.window = K;
    const int per16 = dtype == CIAR_F32 ? 4 : 8;
    p.row_stride = (V + per16 - 1) / per16 * per16;
    return p;
}

static void check_param_validation()
{
    Buf x(1024), ws(1 << 16);
    float o[4];
    ciar_params p = params(64, CIAR_F32, 4);
    auto call = [&](const ciar_params* q) {
        return ciar_quantify(x.p, nullptr, nullptr, 1, q, o, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, ws.p,
                             1 << 16, nullptr);
    };
    EXPECT(call(&p) == CIAR_OK);
    EXPECT(call(nullptr) == CIAR_EINVAL);
    ciar_params q;
    q = p; q.struct_size = 8;            EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.reserved = 1;               EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.dtype = 7;                  EXPECT(call(&q) == CIAR_EUNSUPPORTED);
    q = p; q.vocab = 0;                  EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.vocab = 1 << 20; q.row_stride = 1 << 20; EXPECT(call(&q) == CIAR_EUNSUPPORTED);
    q = p; q.row_stride = 63;            EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.row_stride = 66;            EXPECT(call(&q) == CIAR_EALIGN);
    q = p; q.window = 0;                 EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.radius_max = 17.f;          EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.radius_max = NAN;           EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.tau = INFINITY;             EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.lower_cap = 0.f;            EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.upper_cap = 0.5f;           EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.confidence = 1.f;           EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.radius_scale = INFINITY;    EXPECT(call(&q) == CIAR_EINVAL);
    q = p; q.radius_scale = 0.f;         EXPECT(call(&q) == CIAR_OK);            // radius 0: a = b = 1
    q = p; q.radius_scale = 16.f; q.radius_max = 16.f; EXPECT(call(&q) == CIAR_OK);
    q = p; q.confidence = 1e-6f;         EXPECT(call(&q) == CIAR_OK);
    q = p; q.confidence = 0.9999999f;    EXPECT(call(&q) == CIAR_OK);
    // pointers
    EXPECT(ciar_quantify(nullptr, nullptr, nullptr, 1, &p, o, 0, 0, 0, 0, 0, 0, ws.p, 1 << 16, 0) == CIAR_EINVAL);
    EXPECT(ciar_quantify(x.as<char>() + 4, nullptr, nullptr, 1, &p, o, 0, 0, 0, 0, 0, 0, ws.p, 1 << 16, 0) == CIAR_EALIGN);
    EXPECT(ciar_quantify(x.p, x.as<char>() + 8, nullptr, 1, &p, o, 0, 0, 0, 0, 0, 0, ws.p, 1 << 16, 0) == CIAR_EALIGN);
    EXPECT(ciar_quantify(x.p, nullptr, nullptr, 1, &p, 0, 0, 0, 0, 0, 0, 0, ws.p, 1 << 16, 0) == CIAR_EINVAL);
    EXPECT(ciar_quantify(x.p, nullptr, nullptr, -1, &p, o, 0, 0, 0, 0, 0, 0, ws.p, 1 << 16, 0) == CIAR_EINVAL);
    EXPECT(ciar_quantify(x.p, nullptr, nullptr, (int64_t)1 << 31, &p, o, 0, 0, 0, 0, 0, 0, ws.p, 1 << 16, 0) == CIAR_EUNSUPPORTED);
    EXPECT(ciar_quantify(x.p, nullptr, nullptr, 1, &p, o, 0, 0, 0, 0, 0, 0, nullptr, 0, 0) == CIAR_EWORKSPACE);
    EXPECT(ciar_quantify(x.p, nullptr, nullptr, 1, &p, o, 0, 0, 0, 0, 0, 0, ws.as<char>() + 8, 1 << 15, 0) == CIAR_EALIGN);
    EXPECT(ciar_quantify(x.p, nullptr, nullptr, 1, &p, o, 0, 0, 0, 0, 0, 0, ws.p, 16, 0) == CIAR_EWORKSPACE);
    EXPECT(std::strlen(ciar_last_error()) > 0 && std::strlen(ciar_last_error()) < 512);
    // an empty batch needs nothing and launches nothing
    const int before = stubs::launches;
    EXPECT(ciar_quantify(x.p, nullptr, nullptr, 0, &p, o, 0, 0, 0, 0, 0, 0, nullptr, 0, 0) == CIAR_OK);
    EXPECT(stubs::launches == before);
    // width polynomial: pure host arithmetic
    float coef[4], xm;
    EXPECT(ciar_width_polynomial(&p, coef, &xm) == CIAR_OK && xm > 0.f && xm < 0.25f);
    EXPECT(ciar_width_polynomial(&p, nullptr, &xm) == CIAR_EINVAL);
    for (float kappa : {0.f, 1e-4f, 0.3f, 1.6449f, 5.f, 10.f, 16.f}) {
        q = p; q.radius_scale = kappa; q.radius_max = 16.f;
        EXPECT(ciar_width_polynomial(&q, coef, &xm) == CIAR_OK);
    }
}

// the fused call with every output, all workspace regions written to their full documented extent by the stubs
static void check_fused(int64_t N, int V, int dtype, int K, bool tensor_radius, bool row_outputs, bool static_too = true)
{
    const ciar_params p = params(V, dtype, K);
    const size_t elt = dtype == CIAR_F32 ? 4 : 2, rows = (size_t)N * (size_t)p.row_stride * elt;
    const size_t W = (size_t)((N + K - 1) / K);
    Buf c(rows), t(rows), r(rows), ids(4 * N), ua(4 * N), ur(4 * N);
    Buf lo(4 * N), mid(4 * N), hi(4 * N), om(4 * N), sg(4 * N), sc(4 * N), fl(N), acc(N), rid(4 * N), al(4 * W), rs(4 * W);
    const size_t need = ciar_workspace_bytes(N, &p);
    EXPECT(N == 0 || need >= 113 * (size_t)N);
    Buf ws(need);
    const void* const rad = tensor_radius ? r.p : nullptr;
    int rc = ciar_quantify_verify(c.p, rad, t.p, ids.as<int32_t>(), ua.as<float>(), ur.as<float>(), N, &p, lo.as<float>(),
                                  mid.as<float>(), hi.as<float>(), om.as<float>(), sg.as<float>(), sc.as<float>(),
                                  fl.as<uint8_t>(), row_outputs ? acc.as<uint8_t>() : nullptr,
                                  row_outputs ? rid.as<int32_t>() : nullptr, al.as<int32_t>(), rs.as<int32_t>(), ws.p, need,
                                  nullptr);
    EXPECT(rc == CIAR_OK);
    if (N > 0) {
        const ciar::RowArgs& a = stubs::last_args;
        const char* w0 = ws.as<char>();
        auto inside = [&](const void* q, size_t bytes) {
            return (const char*)q >= w0 && (const char*)q + bytes <= w0 + need;
        };
        EXPECT(inside(a.stats, 88 * (size_t)N));
        EXPECT(inside(a.reject_list, 4 * (size_t)N));
        EXPECT(inside(a.win_words, 16 * (size_t)N));
        EXPECT(((uintptr_t)a.win_words & 127) == 0 && ((uintptr_t)a.stats & 15) == 0);
        if (!row_outputs) { EXPECT(inside(a.accept, (size_t)N)); EXPECT(inside(a.row_id, 4 * (size_t)N)); }
        EXPECT(a.tag != 0 && (a.tag & 0x7fffffffu) != 0);
        EXPECT(a.window == K && a.N == N && a.V == V);
    }
    // verify-only and the two stages on their own
    rc = ciar_verify(c.p, t.p, ids.as<int32_t>(), ua.as<float>(), ur.as<float>(), N, &p, nullptr, nullptr, al.as<int32_t>(),
                     rs.as<int32_t>(), ws.p, need, nullptr);
    EXPECT(rc == CIAR_OK);
    rc = ciar_stream_rows(c.p, rad, t.p, ids.as<int32_t>(), ua.as<float>(), ur.as<float>(), N, &p, lo.as<float>(), 0, 0, 0, 0,
                          sc.as<float>(), 0, acc.as<uint8_t>(), 0, 0, rs.as<int32_t>(), ws.p, need, nullptr);
    EXPECT(rc == CIAR_OK);
    rc = ciar_finish_rows(c.p, rad, t.p, ids.as<int32_t>(), ua.as<float>(), ur.as<float>(), N, &p, lo.as<float>(), 0, 0, 0, 0,
                          sc.as<float>(), 0, acc.as<uint8_t>(), 0, 0, rs.as<int32_t>(), ws.p, need, nullptr);
    EXPECT(rc == CIAR_OK);
    // quantify without drafted ids: tensor mode finds the arg-max tokens into the workspace
    rc = ciar_quantify(c.p, rad, nullptr, N, &p, lo.as<float>(), mid.as<float>(), hi.as<float>(), 0, 0, 0, fl.as<uint8_t>(),
                       ws.p, need, nullptr);
    EXPECT(rc == CIAR_OK);
    if (static_too && N > 0 && N <= CIAR_STATIC_MAX_ROWS) {
        rc = ciar_quantify_verify_static(c.p, rad, t.p, ids.as<int32_t>(), ua.as<float>(), ur.as<float>(), N, &p,
                                         lo.as<float>(), 0, 0, 0, 0, sc.as<float>(), fl.as<uint8_t>(), 0, 0, al.as<int32_t>(),
                                         rs.as<int32_t>(), nullptr);
        EXPECT(rc == CIAR_OK);
    }
    // missing verify inputs
    if (N > 0) {
        EXPECT(ciar_verify(c.p, t.p, nullptr, ua.as<float>(), ur.as<float>(), N, &p, acc.as<uint8_t>(), 0, 0, 0, ws.p, need, 0) == CIAR_EINVAL);
        EXPECT(ciar_verify(c.p, t.p, ids.as<int32_t>(), nullptr, ur.as<float>(), N, &p, acc.as<uint8_t>(), 0, 0, 0, ws.p, need, 0) == CIAR_EINVAL);
        EXPECT(ciar_verify(c.p, nullptr, ids.as<int32_t>(), ua.as<float>(), ur.as<float>(), N, &p, acc.as<uint8_t>(), 0, 0, 0, ws.p, need, 0) == CIAR_EINVAL);
        EXPECT(ciar_verify(c.p, t.p, ids.as<int32_t>(), ua.as<float>(), ur.as<float>(), N, &p, acc.as<uint8_t>(), 0, 0, 0, ws.p, need - 1, 0) == CIAR_EWORKSPACE);
    }
    // the other per-row passes
    Buf sum(4 * N), terms(4 * 7 * N), wts(4 * N), losses(4 * 5);
    EXPECT(ciar_read_rows(c.p, t.p, N, &p, sum.as<float>(), nullptr) == (N >= 0 ? CIAR_OK : CIAR_EINVAL));
    EXPECT(ciar_interdro_loss(c.p, rad, t.p, N, &p, 0.5f, 0.1f, 0.01f, 0.9f, terms.as<float>(), wts.as<float>(),
                              losses.as<float>(), nullptr) == CIAR_OK);
    EXPECT(ciar_window_epilogue(acc.as<uint8_t>(), rid.as<int32_t>(), N, &p, al.as<int32_t>(), rs.as<int32_t>(), nullptr) == CIAR_OK);
    if ((size_t)N * (size_t)p.row_stride <= (1u << 22)) {
        Buf d0(4 * (size_t)N * p.row_stride), d1(4 * (size_t)N * p.row_stride);
        EXPECT(ciar_dense_intervals(c.p, rad, N, &p, d0.as<float>(), nullptr, d1.as<float>(), nullptr) == CIAR_OK);
    }
}

static void check_multihead(int64_t N, int V, int heads, int strategy)
{
    const ciar_params p = params(V, CIAR_F32, 4);
    const int64_t hs = N * p.row_stride + 32;
    Buf c((size_t)heads * hs * 4), r((size_t)heads * hs * 4), ids(4 * N);
    const size_t per = strategy == CIAR_VOTING ? (size_t)heads * N : (size_t)N;
    Buf lo(4 * per), sc(4 * per), fl(N), hf((size_t)heads * N);
    const size_t need = ciar_multihead_workspace_bytes(N, heads, &p);
    Buf ws(need);
    EXPECT(ciar_quantify_multihead(c.p, r.p, heads, hs, ids.as<int32_t>(), N, &p, strategy, lo.as<float>(), 0, 0, 0, 0,
                                   sc.as<float>(), fl.as<uint8_t>(), strategy == CIAR_VOTING ? hf.as<uint8_t>() : nullptr,
                                   ws.p, need, nullptr) == CIAR_OK);
    // flags only: the per-head flags live in the workspace
    EXPECT(ciar_quantify_multihead(c.p, nullptr, heads, hs, nullptr, N, &p, strategy, 0, 0, 0, 0, 0, 0, fl.as<uint8_t>(),
                                   nullptr, ws.p, need, nullptr) == CIAR_OK);
    // tensor radius without ids: arg-max tokens of every head's rows into the workspace
    EXPECT(ciar_quantify_multihead(c.p, r.p, heads, hs, nullptr, N, &p, strategy, lo.as<float>(), 0, 0, 0, 0, 0, 0, nullptr,
                                   ws.p, need, nullptr) == CIAR_OK);
    if (N > 0) {
        EXPECT(ciar_quantify_multihead(c.p, r.p, heads, hs, nullptr, N, &p, strategy, lo.as<float>(), 0, 0, 0, 0, 0, 0, nullptr,
                                       ws.p, need - 1, nullptr) == CIAR_EWORKSPACE);
        EXPECT(ciar_quantify_multihead(c.p, r.p, 0, hs, nullptr, N, &p, strategy, lo.as<float>(), 0, 0, 0, 0, 0, 0, nullptr,
                                       ws.p, need, nullptr) == CIAR_EUNSUPPORTED);
        EXPECT(ciar_quantify_multihead(c.p, r.p, heads, hs, nullptr, N, &p, 5, lo.as<float>(), 0, 0, 0, 0, 0, 0, nullptr, ws.p,
                                       need, nullptr) == CIAR_EINVAL);
        if (heads > 1)
            EXPECT(ciar_quantify_multihead(c.p, r.p, heads, hs - 40, nullptr, N, &p, strategy, lo.as<float>(), 0, 0, 0, 0, 0, 0,
                                           nullptr, ws.p, need, nullptr) == CIAR_EINVAL);
    }
}

static void check_interhead(int64_t N, int V, int D)
{
    const ciar_params p = params(V, CIAR_F32, 4);
    Buf h(2 * (size_t)N * D), w(2 * 2 * (size_t)V * D), b(4 * 2 * (size_t)V), ids(4 * N), sc(4 * N), fl(N);
    const size_t need = ciar_interhead_workspace_bytes(N, &p);
    Buf ws(need), ce(4 * (size_t)N * p.row_stride), ra(4 * (size_t)N * p.row_stride);
    EXPECT(ciar_interhead_logits(h.p, w.p, b.as<float>(), D, N, &p, ce.as<float>(), ra.as<float>(), nullptr) == CIAR_OK);
    EXPECT(ciar_interhead_quantify(h.p, w.p, nullptr, D, ids.as<int32_t>(), N, &p, 0, 0, 0, 0, 0, sc.as<float>(),
                                   fl.as<uint8_t>(), ws.p, need, nullptr) == CIAR_OK);
    if (N > 0) {
        EXPECT(stubs::last_head.row_tiles == (N + ciar::kHeadTileRows - 1) / ciar::kHeadTileRows);
        EXPECT(ciar_interhead_quantify(h.p, w.p, nullptr, D, ids.as<int32_t>(), N, &p, 0, 0, 0, 0, 0, sc.as<float>(),
                                       fl.as<uint8_t>(), ws.p, need - 1, nullptr) == CIAR_EWORKSPACE);
        EXPECT(ciar_interhead_logits(h.p, w.p, nullptr, D + 8, N, &p, ce.as<float>(), ra.as<float>(), nullptr) == CIAR_EUNSUPPORTED);
        EXPECT(ciar_interhead_logits(h.p, w.p, nullptr, D, N, &p, nullptr, ra.as<float>(), nullptr) == CIAR_EINVAL);
        ciar_params q = p; q.vocab = V + 4; q.row_stride = V + 4;
        EXPECT(ciar_interhead_logits(h.p, w.p, nullptr, D, N, &q, ce.as<float>(), ra.as<float>(), nullptr) == CIAR_EUNSUPPORTED);
        q = p; q.dtype = CIAR_BF16;
        EXPECT(ciar_interhead_logits(h.p, w.p, nullptr, D, N, &q, ce.as<float>(), ra.as<float>(), nullptr) == CIAR_EUNSUPPORTED);
    }
}

int main()
{
    {   // the first look-ups of the built-in scratch buffer, from several threads at once (the calls stop at the
        // parameter check that follows the look-up, so nothing is written to the shared buffer)
        std::vector<std::thread> first;
        for (int t = 0; t < 4; ++t)
            first.emplace_back([] {
                ciar_params p = params(8, CIAR_F32, 8);
                p.window = 0;
                Buf x(64);
                float o;
                for (int i = 0; i < 50; ++i)
                    EXPECT(ciar_quantify_verify_static(x.p, 0, x.p, x.as<int32_t>(), x.as<float>(), x.as<float>(), 2, &p, &o,
                                                       0, 0, 0, 0, 0, 0, 0, 0, 0, 0, nullptr) == CIAR_EINVAL);
            });
        for (auto& th : first) th.join();
    }
    check_param_validation();
    for (int64_t N : {0, 1, 7, 8, 9, 127, 128, 129, 1000, 4097})
        for (int K : {1, 3, 8, 300})
            for (int tr = 0; tr < 2; ++tr) {
                check_fused(N, 37, CIAR_F32, K, tr, N % 2);
                check_fused(N, 1000, CIAR_BF16, K, tr, !(N % 2));
            }
    check_fused(CIAR_STATIC_MAX_ROWS, 8, CIAR_F32, 8, false, false);
    {   // one row more than the built-in buffer holds
        const ciar_params p = params(8, CIAR_F32, 8);
        Buf x(64);
        float o;
        EXPECT(ciar_quantify_verify_static(x.p, 0, x.p, x.as<int32_t>(), x.as<float>(), x.as<float>(),
                                           CIAR_STATIC_MAX_ROWS + 1, &p, &o, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, nullptr) == CIAR_EWORKSPACE);
    }
    for (int64_t N : {0, 1, 17, 513})
        for (int heads : {1, 2, 5, 8})
            for (int s : {CIAR_VOTING, CIAR_ENSEMBLE}) check_multihead(N, 130, heads, s);
    for (int64_t N : {0, 1, 127, 129, 300}) check_interhead(N, 256, 128);

    // concurrent callers: the error text is per thread, the tags are shared (calls on the built-in scratch buffer are
    // documented to race when they overlap, so they stay out of this part)
    std::vector<std::thread> pool;
    for (int t = 0; t < 4; ++t)
        pool.emplace_back([t] {
            for (int i = 0; i < 20; ++i) {
                check_fused(64 + t, 37, CIAR_F32, 4, i & 1, false, false);
                ciar_params p = params(64, CIAR_F32, 4);
                p.window = -t;
                float o;
                Buf x(256);
                EXPECT(ciar_quantify(x.p, 0, 0, 1, &p, &o, 0, 0, 0, 0, 0, 0, x.p, 256, 0) == CIAR_EINVAL);
                char want[64];
                std::snprintf(want, sizeof want, "(got %d)", -t);
                EXPECT(std::strstr(ciar_last_error(), want) != nullptr);
            }
        });
    for (auto& th : pool) th.join();

    std::printf("%d launches, %d failed expectations\n", (int)stubs::launches, g_failed);
    return g_failed ? 1 : 0;
}
