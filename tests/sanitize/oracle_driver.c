/* Runs every entry point of the oracle on small seeded inputs that reach its edges (one token, ragged windows, an
 * empty batch, rows of equal logits, huge and tiny logits, radii at the clamp, uniforms at 0 and just below 1);
 * built together with oracle/ciar_oracle.c under AddressSanitizer and UndefinedBehaviorSanitizer by
 * tests/test_sanitizers.py.  Every buffer has exactly the documented size, so an index mistake in the oracle is a
 * heap overflow.  The values are not judged here (the pins do that), only that they are finite where they must be:
 * exit status 0 means the sanitizers saw nothing. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/ciar_oracle.c"

static uint64_t g_state = 0x9e3779b97f4a7c15ull;
static double uniform01(void)
{
    g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
    return (double)(g_state >> 11) / 9007199254740992.0;
}

static int g_failed = 0;
#define EXPECT(c) do { if (!(c)) { fprintf(stderr, "%s:%d: EXPECT(%s) failed\n", __FILE__, __LINE__, #c); ++g_failed; } } while (0)

static void* exact(size_t bytes) { void* p = malloc(bytes ? bytes : 1); if (!p) abort(); return p; }

static uint16_t to_bf16(float f) { uint32_t b; memcpy(&b, &f, 4); return (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16); }

/* kind: 0 = gaussian-like rows, 1 = all logits equal, 2 = one dominant token, 3 = logits of magnitude 80 */
static void* make_rows(int64_t rows, const ciar_oracle_params* P, int kind, double scale)
{
    const size_t elt = P->dtype == 0 ? 4 : (P->dtype == 1 ? 2 : 8);
    char* base = (char*)exact((size_t)rows * (size_t)P->row_stride * elt);
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t i = 0; i < P->row_stride; ++i) {
            double v = scale * (uniform01() + uniform01() + uniform01() - 1.5) * 2.0;
            if (kind == 1) v = 0.25;
            if (kind == 2 && i == (r * 7) % P->vocab) v += 30.0;
            if (kind == 3) v = (i & 1) ? 80.0 + v : -80.0 + v;
            const int64_t k = r * P->row_stride + i;
            if (P->dtype == 0) ((float*)base)[k] = (float)v;
            else if (P->dtype == 1) ((uint16_t*)base)[k] = to_bf16((float)v);
            else ((double*)base)[k] = v;
        }
    return base;
}

static void run_case(int64_t N, int V, int dtype, int K, int kind, int tensor_radius, double kappa, double rmax, int normalize,
                     int threads)
{
    ciar_oracle_params P;
    memset(&P, 0, sizeof P);
    P.vocab = V; P.dtype = dtype; P.row_stride = V + (V % 3);
    P.kappa = kappa; P.confidence = 0.9; P.radius_max = rmax; P.tau = 0.3;
    P.lower_cap = 0.99; P.upper_cap = 1.01; P.normalize = normalize; P.window = K;
    const int64_t W = (N + K - 1) / K;
    void* c = make_rows(N, &P, kind, 2.0);
    void* t = make_rows(N, &P, kind == 1 ? 0 : kind, 2.5);
    void* r = make_rows(N, &P, 0, 3.0);
    int32_t* ids = (int32_t*)exact(4 * (size_t)N);
    float* ua = (float*)exact(4 * (size_t)N); float* ur = (float*)exact(4 * (size_t)N);
    for (int64_t i = 0; i < N; ++i) {
        ids[i] = (int32_t)(uniform01() * V) % V;
        ua[i] = i % 5 == 0 ? 0.f : (i % 5 == 1 ? 0.99999994f : (float)uniform01());
        ur[i] = i % 7 == 0 ? 0.f : (i % 7 == 1 ? 0.99999994f : (float)uniform01());
    }
    double* q[6];
    for (int j = 0; j < 6; ++j) q[j] = (double*)exact(8 * (size_t)N);
    uint8_t* flags = (uint8_t*)exact((size_t)N);
    EXPECT(ciar_oracle_quantify(c, tensor_radius ? r : NULL, ids, N, &P, q[0], q[1], q[2], q[3], q[4], q[5], flags, threads) == 0);
    for (int64_t i = 0; i < N; ++i) {
        EXPECT(q[0][i] >= 0.0 && q[0][i] <= q[1][i] * (1 + 1e-12) && q[1][i] <= q[2][i] * (1 + 1e-12));
        EXPECT(isfinite(q[3][i]) && isfinite(q[4][i]) && isfinite(q[5][i]) && flags[i] <= 1);
    }
    EXPECT(ciar_oracle_quantify(c, tensor_radius ? r : NULL, NULL, N, &P, q[0], NULL, q[2], NULL, NULL, q[5], NULL, threads) == 0);

    uint8_t* acc = (uint8_t*)exact((size_t)N); int32_t* rid = (int32_t*)exact(4 * (size_t)N);
    int32_t* al = (int32_t*)exact(4 * (size_t)W); int32_t* rs = (int32_t*)exact(4 * (size_t)W);
    double* lr = (double*)exact(8 * (size_t)N); double* rm = (double*)exact(8 * (size_t)N);
    EXPECT(ciar_oracle_verify(c, t, ids, ua, ur, N, &P, acc, rid, al, rs, lr, rm, threads) == 0);
    for (int64_t w = 0; w < W; ++w) {
        const int64_t len = (w + 1) * K <= N ? K : N - w * K;
        EXPECT(al[w] >= 0 && al[w] <= len);
        EXPECT((al[w] == len) == (rs[w] == -1));
        EXPECT(rs[w] >= -1 && rs[w] < V);
    }
    EXPECT(ciar_oracle_verify(c, t, ids, ua, ur, N, &P, acc, NULL, al, NULL, NULL, NULL, threads) == 0);
    if (N > 0) {
        double* cdf = (double*)exact(8 * (size_t)V);
        const double R = ciar_oracle_residual_cdf(c, t, N - 1, &P, cdf);
        EXPECT(R >= 0.0 && R <= 1.0 + 1e-12);
        free(cdf);
    }

    if ((size_t)N * (size_t)V <= 200000) {
        double* d[3];
        for (int j = 0; j < 3; ++j) d[j] = (double*)exact(8 * (size_t)N * (size_t)V);
        EXPECT(ciar_oracle_dense_intervals(c, tensor_radius ? r : NULL, N, &P, d[0], d[1], d[2]) == 0);
        for (int j = 0; j < 3; ++j) free(d[j]);
    }
    double* terms = (double*)exact(8 * 7 * (size_t)N); double* wts = (double*)exact(8 * (size_t)N); double losses[5];
    EXPECT(ciar_oracle_interdro_loss(c, tensor_radius ? r : NULL, t, N, &P, 0.5, 0.1, 0.01, 0.9, terms, wts, losses, threads) == 0);
    if (N > 0) for (int j = 0; j < 5; ++j) EXPECT(isfinite(losses[j]));

    free(terms); free(wts); free(acc); free(rid); free(al); free(rs); free(lr); free(rm); free(flags);
    for (int j = 0; j < 6; ++j) free(q[j]);
    free(ids); free(ua); free(ur); free(c); free(t); free(r);
}

static void run_heads(int64_t N, int V, int heads, int strategy, int tensor_radius)
{
    ciar_oracle_params P;
    memset(&P, 0, sizeof P);
    P.vocab = V; P.dtype = 0; P.row_stride = V + 1;
    P.kappa = 1.0; P.confidence = 0.9; P.radius_max = 10.0; P.tau = 0.3;
    P.lower_cap = 0.99; P.upper_cap = 1.01; P.normalize = 1; P.window = 4;
    const int64_t hs = N * P.row_stride;                       /* heads back to back */
    void* c = make_rows((int64_t)heads * N, &P, 0, 2.0);
    void* r = make_rows((int64_t)heads * N, &P, 0, 1.0);
    int32_t* ids = (int32_t*)exact(4 * (size_t)N);
    for (int64_t i = 0; i < N; ++i) ids[i] = (int32_t)(uniform01() * V) % V;
    const size_t per = strategy == 0 ? (size_t)heads * (size_t)N : (size_t)N;
    double* q[6];
    for (int j = 0; j < 6; ++j) q[j] = (double*)exact(8 * per);
    uint8_t* flags = (uint8_t*)exact((size_t)N); uint8_t* hf = (uint8_t*)exact((size_t)heads * (size_t)N);
    EXPECT(ciar_oracle_quantify_multihead(c, tensor_radius ? r : NULL, heads, hs, ids, N, &P, strategy, q[0], q[1], q[2], q[3], q[4],
                                          q[5], flags, strategy == 0 ? hf : NULL, 2) == 0);
    EXPECT(ciar_oracle_quantify_multihead(c, tensor_radius ? r : NULL, heads, hs, NULL, N, &P, strategy, q[0], q[1], q[2], q[3], q[4],
                                          q[5], flags, strategy == 0 ? hf : NULL, 1) == 0);
    for (int j = 0; j < 6; ++j) free(q[j]);
    free(flags); free(hf); free(ids); free(c); free(r);
}

int main(void)
{
    EXPECT(fabs(ciar_oracle_kappa(0.9) - 1.6448536269514722) < 1e-9);
    const int64_t Ns[] = {0, 1, 5, 8, 13};
    const int Vs[] = {1, 2, 3, 64, 65, 1000};
    for (int a = 0; a < 5; ++a)
        for (int b = 0; b < 6; ++b)
            for (int kind = 0; kind < 4; ++kind)
                for (int tr = 0; tr < 2; ++tr) {
                    run_case(Ns[a], Vs[b], 0, 4, kind, tr, -1.0, 10.0, 1, 1 + (a & 1));
                    run_case(Ns[a], Vs[b], 1, 3, kind, tr, 1.0, 10.0, 1, 2);
                    run_case(Ns[a], Vs[b], 2, 1, kind, tr, 16.0, 16.0, kind & 1, 1);
                    run_case(Ns[a], Vs[b], 0, 300, kind, tr, 0.0, 0.0, 1, 3);
                }
    for (int heads = 1; heads <= 5; heads += 2)
        for (int s = 0; s < 2; ++s)
            for (int tr = 0; tr < 2; ++tr) { run_heads(0, 33, heads, s, tr); run_heads(9, 33, heads, s, tr); run_heads(4, 1, heads, s, tr); }
    printf("%d failed expectations\n", g_failed);
    return g_failed ? 1 : 0;
}
