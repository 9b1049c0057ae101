/*
 * CIAR quantify + verify -- reference oracle (TEST INFRASTRUCTURE, not product code).
 *
 * A plain, slow, fp64 CPU evaluation of what the device-side self-verification pass
 * of CIAR computes for every drafted image-token position, written from the paper:
 *
 *   - softmax of the centre logits with the max-trick      (Sec. 3.2.3 "p = softmax(o)";
 *                                                            App. "Proof of Interval Validity", last paragraph)
 *   - InterFuse lower / upper probability bounds            (App. "Proof of Interval Validity", the two
 *                                                            equations that define p^l_i and p^u_i)
 *   - the 0.99 / 1.01 normalisation of the bounds           (same appendix, the two scaling equations)
 *   - widths delta, Total Ambiguity Omega, Confidence
 *     Disparity Sigma (population std), score U = Omega*Sigma (Eq. "uncertainty_score"; App. "Analysis of the
 *                                                            Uncertainty Quantification", first three equations)
 *   - the threshold rule  "accept locally iff U <= tau"     (Algorithm 1, the test on U_t)
 *   - aggregation of several Interval Heads                 (Sec. 4, ablation on the Inter-Head: "Voting" = the
 *                                                            majority of the heads' decisions, "Ensemble" = the
 *                                                            heads' probability distributions averaged)
 *   - the forward value of the Inter-DRO training loss      (Sec. 3.2.3 "Interval-enhanced Distributionally Robust
 *                                                            Training": anchor, DRO and alignment equations)
 *   - cloud verification of a window of K drafted tokens and resampling (Algorithm 1, the "Cloud verification"
 *     step and the following resample / advance steps).  The paper names this step as speculative decoding
 *     (Introduction) without writing the test down; this file uses the standard speculative-sampling rule:
 *     accept x ~ p with probability min(1, q(x)/p(x)), otherwise draw from (q - p)^+ / ||(q - p)^+||_1,
 *     p = softmax(centre logits), q = softmax(target logits).
 *
 * Every sum runs sequentially in index order, in double precision.  There is no blocking,
 * no fusion and no reordering (one sum is taken twice, with and without its largest term: see row_rest).  Only tests/, __graft_entry__.smoke() and the cpu_baseline
 * leg of bench.py may call this file; the product path never does.  It shares no code with
 * the HIP kernels.
 *
 * The Interval Head's two linear maps that produce the centre and raw-radius logits (Sec. 3.2.1, "Interval Head
 * Architecture") are evaluated by the Python front end (numpy's fp64 matrix product); their fp64 logits enter the
 * functions here through the float64 logit type.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py (library softmax,
 * logistic sigmoid for V = 2, closed forms for uniform and one-hot rows, the appendix's
 * claims and propositions, brute-force enumeration of the acceptance law for V <= 8).
 *
 * Parameters not fixed by the paper (stated as readings where this repo documents them):
 *   - kappa: the scale of the logit half-width.  It is either given directly or derived from an
 *     "interval confidence" gamma as the two-sided standard-normal quantile
 *     kappa = sqrt(2) * erfinv(gamma).
 *   - radius_max: the clamp on the radius (the paper clamps but gives no value).
 *   - the radius itself: r_i = min(kappa * rho_i, radius_max).  Scalar mode (no radius tensor): rho_i = 1.
 *     Tensor mode: rho_i = Softplus(raw_i) for the raw output raw of the radius half of the Interval Head
 *     (Sec. 3.2.3, the equation that defines c_t and r_t); kappa = 1 is the paper's head as written.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct ciar_oracle_params {
    int32_t vocab;        /* V >= 1 */
    int32_t dtype;        /* 0 = float32 logits, 1 = bfloat16 logits (raw uint16), 2 = float64 logits */
    int64_t row_stride;   /* elements between consecutive rows, >= V */
    double  kappa;        /* scalar logit radius before the clamp; if < 0 it is derived from confidence */
    double  confidence;   /* gamma in (0,1), used only when kappa < 0 */
    double  radius_max;   /* clamp on the radius */
    double  tau;          /* threshold on U */
    double  lower_cap;    /* 0.99 in the paper */
    double  upper_cap;    /* 1.01 in the paper */
    int32_t normalize;    /* 1 = apply the caps, 0 = raw InterFuse */
    int32_t window;       /* K >= 1: drafted tokens per cloud verification call */
} ciar_oracle_params;

/* ---- input widening ------------------------------------------------------------------ */

static double load_logit(const void* base, int32_t dtype, int64_t index)
{
    if (dtype == 0) {
        return (double)((const float*)base)[index];
    } else if (dtype == 2) {
        /* logits already in double precision (the Interval Head's linear maps evaluated in fp64) */
        return ((const double*)base)[index];
    } else {
        /* bfloat16 is the upper half of an IEEE float32: widening is exact. */
        uint32_t bits = ((uint32_t)((const uint16_t*)base)[index]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* ---- radius ------------------------------------------------------------------------- */

/* kappa(gamma) = sqrt(2) * erfinv(gamma): the z with P(|Z| <= z) = gamma for Z ~ N(0,1).
 * Solved by bisection on erf (monotone), which needs no inverse-erf routine. */
double ciar_oracle_kappa(double gamma)
{
    if (!(gamma > 0.0)) return 0.0;
    if (!(gamma < 1.0)) return INFINITY;
    double lo = 0.0, hi = 40.0;
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (erf(mid / sqrt(2.0)) < gamma) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

/* Softplus(x) = ln(1 + e^x), evaluated on the side that cannot overflow. */
static double softplus(double x)
{
    return x > 0.0 ? x + log1p(exp(-x)) : log1p(exp(x));
}

/* The radius scale: given, or the quantile of the interval confidence. */
static double radius_scale(const ciar_oracle_params* P)
{
    return P->kappa >= 0.0 ? P->kappa : ciar_oracle_kappa(P->confidence);
}

/* r_i = min(kappa * rho_i, radius_max); rho_i = 1 without a radius tensor, else Softplus(raw_i). */
static double token_radius(const ciar_oracle_params* P, double kappa, const void* radius, int64_t index)
{
    const double rho = radius ? softplus(load_logit(radius, P->dtype, index)) : 1.0;
    const double r = kappa * rho;
    return r < P->radius_max ? r : P->radius_max;
}

/* ---- one row of the quantifier -------------------------------------------------------- */

/* What row_interfuse needs besides S: sum_{j != i} e[j].  For every token but the largest this is S - e[i]
 * (e[i] <= S / 2: nothing cancels).  For the largest token S - e[i] would cancel -- when it holds nearly all of
 * the mass, S has already dropped what lies below half an ulp of it -- so its sum over the others is formed
 * directly. */
typedef struct {
    int    imax;        /* lowest index of the largest e[i] */
    double rest_imax;   /* sum_{j != imax} e[j], summed in index order without e[imax] */
} row_rest;

/* Fills e[i] = exp(c_i - max c) and returns S = sum_i e[i]; *m_out = max c; *rest (may be NULL) as above. */
static double row_exponentials_ext(const void* logits, const ciar_oracle_params* P, int64_t row,
                                   double* e, double* m_out, row_rest* rest)
{
    const int64_t off = row * P->row_stride;
    const int V = P->vocab;
    double m = -INFINITY;
    int imax = 0;
    for (int i = 0; i < V; ++i) {
        double c = load_logit(logits, P->dtype, off + i);
        if (c > m) { m = c; imax = i; }
    }
    double S = 0.0, others = 0.0;
    for (int i = 0; i < V; ++i) {
        double c = load_logit(logits, P->dtype, off + i);
        e[i] = exp(c - m);
        S += e[i];
        if (i != imax) others += e[i];
    }
    *m_out = m;
    if (rest) { rest->imax = imax; rest->rest_imax = others; }
    return S;
}

static double row_exponentials(const void* logits, const ciar_oracle_params* P, int64_t row,
                               double* e, double* m_out)
{
    return row_exponentials_ext(logits, P, row, e, m_out, NULL);
}

/* InterFuse bounds for the whole row, normalised if requested.
 * In: e[i], S and the sum over the others of the largest token (see row_rest), the raw radius tensor (NULL:
 * scalar mode) and the row.  Out: pl[i], pu[i] (the final, possibly scaled, bounds).
 * The appendix prints the denominators as S - e_i + e_i e^{-/+ r_i}; S - e_i equals the sum over the other tokens,
 * which is what row_rest forms directly for the largest token (the one token for which the subtraction cancels). */
static void row_interfuse(const double* e, double S, const row_rest* rest, const ciar_oracle_params* P,
                          const void* radius, int64_t row, double* pl, double* pu)
{
    const int V = P->vocab;
    const double kappa = radius_scale(P);
    double Sl = 0.0, Su = 0.0;
    for (int i = 0; i < V; ++i) {
        const double r = token_radius(P, kappa, radius, row * P->row_stride + i);
        double down = e[i] * exp(-r);   /* exp(c_i - r_i) up to the common shift */
        double up   = e[i] * exp(r);    /* exp(c_i + r_i) up to the common shift */
        const double others = i == rest->imax ? rest->rest_imax : S - e[i];   /* sum over the other tokens */
        pl[i] = down / (others + down);
        pu[i] = up / (others + up);
        Sl += pl[i];
        Su += pu[i];
    }
    if (P->normalize) {
        double fl = P->lower_cap / Sl; if (fl > 1.0) fl = 1.0;   /* min(1, 0.99/S_l) */
        double fu = P->upper_cap / Su; if (fu < 1.0) fu = 1.0;   /* max(1, 1.01/S_u) */
        for (int i = 0; i < V; ++i) { pl[i] *= fl; pu[i] *= fu; }
    }
}

static int lowest_argmax(const double* x, int V)
{
    int k = 0;
    for (int i = 1; i < V; ++i) if (x[i] > x[k]) k = i;
    return k;
}

/*
 * Quantifier for rows [0, N).  Outputs are fp64; any output pointer may be NULL.
 *   radius == NULL: scalar radius; else the raw radius tensor, same dtype and row stride as draft.
 *   ids == NULL: the reported token is the lowest-index argmax of the centre logits.
 *   flags[i] = 1 means "uncertain, send to the cloud" = (U > tau); U == tau is not flagged.
 * Returns 0, or -1 on allocation failure.
 */
int ciar_oracle_quantify(const void* draft, const void* radius, const int32_t* ids, int64_t N,
                         const ciar_oracle_params* P,
                         double* p_lo, double* p_mid, double* p_hi,
                         double* omega, double* sigma, double* score, uint8_t* flags,
                         int threads)
{
    const int V = P->vocab;
    int failed = 0;
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
    {
        double* e  = (double*)malloc(sizeof(double) * (size_t)V);
        double* pl = (double*)malloc(sizeof(double) * (size_t)V);
        double* pu = (double*)malloc(sizeof(double) * (size_t)V);
        if (!e || !pl || !pu) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (int64_t row = 0; row < N; ++row) {
                double m;
                row_rest rest;
                double S = row_exponentials_ext(draft, P, row, e, &m, &rest);
                row_interfuse(e, S, &rest, P, radius, row, pl, pu);

                /* widths, L1 norm, population standard deviation (two passes) */
                double Om = 0.0;
                for (int i = 0; i < V; ++i) Om += pu[i] - pl[i];
                double mean = Om / (double)V;
                double ss = 0.0;
                for (int i = 0; i < V; ++i) {
                    double d = (pu[i] - pl[i]) - mean;
                    ss += d * d;
                }
                double Sg = sqrt(ss / (double)V);
                double U = Om * Sg;

                int x = ids ? ids[row] : lowest_argmax(e, V);
                if (p_lo)  p_lo[row]  = pl[x];
                if (p_mid) p_mid[row] = e[x] / S;
                if (p_hi)  p_hi[row]  = pu[x];
                if (omega) omega[row] = Om;
                if (sigma) sigma[row] = Sg;
                if (score) score[row] = U;
                if (flags) flags[row] = (uint8_t)(U > P->tau);
            }
        }
        free(e); free(pl); free(pu);
    }
    return failed ? -1 : 0;
}

/* Dense export of the three per-token curves, [N, V] each, for tests. */
int ciar_oracle_dense_intervals(const void* draft, const void* radius, int64_t N,
                                const ciar_oracle_params* P, double* p_lo, double* p_mid, double* p_hi)
{
    const int V = P->vocab;
    double* e = (double*)malloc(sizeof(double) * (size_t)V);
    if (!e) return -1;
    for (int64_t row = 0; row < N; ++row) {
        double m;
        row_rest rest;
        double S = row_exponentials_ext(draft, P, row, e, &m, &rest);
        row_interfuse(e, S, &rest, P, radius, row, p_lo + row * (int64_t)V, p_hi + row * (int64_t)V);
        for (int i = 0; i < V; ++i) p_mid[row * (int64_t)V + i] = e[i] / S;
    }
    free(e);
    return 0;
}

/* ---- several heads ------------------------------------------------------------------- */

static const void* head_base(const void* base, int32_t dtype, int64_t head, int64_t head_stride)
{
    if (!base) return NULL;
    return (const char*)base + (size_t)head * (size_t)head_stride * (dtype == 0 ? 4u : dtype == 2 ? 8u : 2u);
}

/*
 * Quantifier over H heads.  draft (and radius, unless NULL) hold H tensors [N, row_stride], head h starting
 * head_stride elements after head h-1.  The paper names the two strategies without formulas (Sec. 4, ablation
 * on the Inter-Head); the readings used here:
 *
 *   strategy 0, Voting:   every head runs the quantifier on its own; the voted flag is the strict majority of
 *                         the heads' flags (2 * votes > H).  p_lo ... score are per head, [H, N];
 *                         head_flags [H, N]; flags [N] is the vote.
 *   strategy 1, Ensemble: the heads' curves are averaged token by token -- pl_i = mean_h pl_{h,i},
 *                         p_i = mean_h p_{h,i}, pu_i = mean_h pu_{h,i}, every head after its own 0.99 / 1.01
 *                         scaling -- and widths, Omega, Sigma, U and the flag follow from the averaged
 *                         curves.  All outputs are [N]; head_flags is not written.  ids == NULL reports the
 *                         lowest-index arg-max of the averaged p.
 * Returns 0, or -1 on allocation failure / unknown strategy.
 */
int ciar_oracle_quantify_multihead(const void* draft, const void* radius, int32_t heads, int64_t head_stride,
                                   const int32_t* ids, int64_t N, const ciar_oracle_params* P, int32_t strategy,
                                   double* p_lo, double* p_mid, double* p_hi,
                                   double* omega, double* sigma, double* score,
                                   uint8_t* flags, uint8_t* head_flags, int threads)
{
    const int V = P->vocab;
    const int H = heads;
    if (H < 1) return -1;
    if (strategy == 0) {
        uint8_t* hf = (uint8_t*)malloc((size_t)H * (size_t)(N > 0 ? N : 1));
        if (!hf) return -1;
        for (int h = 0; h < H; ++h) {
            const int64_t o = (int64_t)h * N;
            int rc = ciar_oracle_quantify(head_base(draft, P->dtype, h, head_stride),
                                          head_base(radius, P->dtype, h, head_stride), ids, N, P,
                                          p_lo ? p_lo + o : NULL, p_mid ? p_mid + o : NULL, p_hi ? p_hi + o : NULL,
                                          omega ? omega + o : NULL, sigma ? sigma + o : NULL,
                                          score ? score + o : NULL, hf + o, threads);
            if (rc) { free(hf); return rc; }
        }
        for (int64_t row = 0; row < N; ++row) {
            int votes = 0;
            for (int h = 0; h < H; ++h) votes += hf[(int64_t)h * N + row];
            if (flags) flags[row] = (uint8_t)(2 * votes > H);
        }
        if (head_flags) memcpy(head_flags, hf, (size_t)H * (size_t)N);
        free(hf);
        return 0;
    }
    if (strategy != 1) return -1;

    int failed = 0;
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
    {
        double* e   = (double*)malloc(sizeof(double) * (size_t)V);
        double* pl  = (double*)malloc(sizeof(double) * (size_t)V);
        double* pu  = (double*)malloc(sizeof(double) * (size_t)V);
        double* apl = (double*)malloc(sizeof(double) * (size_t)V);
        double* apm = (double*)malloc(sizeof(double) * (size_t)V);
        double* apu = (double*)malloc(sizeof(double) * (size_t)V);
        if (!e || !pl || !pu || !apl || !apm || !apu) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (int64_t row = 0; row < N; ++row) {
                for (int i = 0; i < V; ++i) apl[i] = apm[i] = apu[i] = 0.0;
                for (int h = 0; h < H; ++h) {
                    const void* c = head_base(draft, P->dtype, h, head_stride);
                    const void* r = head_base(radius, P->dtype, h, head_stride);
                    double m;
                    row_rest rest;
                    double S = row_exponentials_ext(c, P, row, e, &m, &rest);
                    row_interfuse(e, S, &rest, P, r, row, pl, pu);
                    for (int i = 0; i < V; ++i) { apl[i] += pl[i]; apm[i] += e[i] / S; apu[i] += pu[i]; }
                }
                for (int i = 0; i < V; ++i) { apl[i] /= (double)H; apm[i] /= (double)H; apu[i] /= (double)H; }

                double Om = 0.0;
                for (int i = 0; i < V; ++i) Om += apu[i] - apl[i];
                double mean = Om / (double)V;
                double ss = 0.0;
                for (int i = 0; i < V; ++i) {
                    double d = (apu[i] - apl[i]) - mean;
                    ss += d * d;
                }
                double Sg = sqrt(ss / (double)V);
                double U = Om * Sg;

                int x = ids ? ids[row] : lowest_argmax(apm, V);
                if (p_lo)  p_lo[row]  = apl[x];
                if (p_mid) p_mid[row] = apm[x];
                if (p_hi)  p_hi[row]  = apu[x];
                if (omega) omega[row] = Om;
                if (sigma) sigma[row] = Sg;
                if (score) score[row] = U;
                if (flags) flags[row] = (uint8_t)(U > P->tau);
            }
        }
        free(e); free(pl); free(pu); free(apl); free(apm); free(apu);
    }
    return failed ? -1 : 0;
}

/* ---- Inter-DRO loss, forward ----------------------------------------------------------- */

/* ln softmax(o)_i for a row of V logits o (fp64): lsm[i] = o_i - max o - ln sum_j exp(o_j - max o). */
static void log_softmax(const double* o, int V, double* lsm)
{
    double m = -INFINITY;
    for (int i = 0; i < V; ++i) if (o[i] > m) m = o[i];
    double s = 0.0;
    for (int i = 0; i < V; ++i) s += exp(o[i] - m);
    const double lz = m + log(s);
    for (int i = 0; i < V; ++i) lsm[i] = o[i] - lz;
}

/*
 * Forward value of the Inter-DRO loss (Sec. 3.2.3, the four loss equations) for a batch of N rows.
 *   p_mid = softmax(c), p_up = softmax(c + r), p_lo = softmax(c - r), p_cloud = softmax(cloud), r_i as in the
 *   quantifier (min(kappa * rho_i, radius_max), rho_i = Softplus(raw_i) with a radius tensor, else 1);
 *   L1(p) = ||p - p_cloud||_1,  CE(p) = - sum_i p_cloud,i ln p_i,  KL = sum_i p_cloud,i (ln p_cloud,i - ln p_mid,i)
 *   (tokens with p_cloud,i = 0 contribute nothing to CE and KL);
 *   w_n = exp(alpha CE_n(p_lo)) / sum_k exp(alpha CE_k(p_lo)),  DRO = sum_n w_n CE_n(p_lo).
 * Per-row terms rows[t * N + n], t = 0..6: L1(p_mid), L1(p_up), L1(p_lo), CE(p_mid), CE(p_up), CE(p_lo), KL.
 * losses[0..4] = centre, upper, lower, DRO, total, with the batch reduction the paper leaves open taken as the
 * mean over the N rows for the anchor and alignment terms (the DRO term is the weighted sum as printed):
 *   centre = mean(lambda_v L1(p_mid) + lambda_p CE(p_mid) + lambda_beta KL)
 *   upper  = mean(lambda_v L1(p_up) + lambda_p CE(p_up)),   lower = mean(lambda_v L1(p_lo) + lambda_p CE(p_lo))
 *   total  = centre + upper + lower + DRO.
 * Any of rows, weights, losses may be NULL.  Returns 0, or -1 on allocation failure.
 */
int ciar_oracle_interdro_loss(const void* center, const void* radius, const void* cloud, int64_t N,
                              const ciar_oracle_params* P, double lambda_v, double lambda_p, double lambda_beta,
                              double alpha, double* rows, double* weights, double* losses, int threads)
{
    const int V = P->vocab;
    int failed = 0;
    if (threads < 1) threads = 1;
    double* terms = (double*)malloc(sizeof(double) * 7 * (size_t)(N > 0 ? N : 1));
    if (!terms) return -1;
#pragma omp parallel num_threads(threads)
    {
        double* o   = (double*)malloc(sizeof(double) * (size_t)V);
        double* lpc = (double*)malloc(sizeof(double) * (size_t)V);
        double* lp  = (double*)malloc(sizeof(double) * (size_t)V);
        double* r   = (double*)malloc(sizeof(double) * (size_t)V);
        if (!o || !lpc || !lp || !r) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
            const double kappa = radius_scale(P);
#pragma omp for schedule(static)
            for (int64_t n = 0; n < N; ++n) {
                const int64_t off = n * P->row_stride;
                for (int i = 0; i < V; ++i) {
                    o[i] = load_logit(cloud, P->dtype, off + i);
                    r[i] = token_radius(P, kappa, radius, off + i);
                }
                log_softmax(o, V, lpc);
                for (int v = 0; v < 3; ++v) {                      /* mid, up, lo */
                    const double sgn = v == 0 ? 0.0 : (v == 1 ? 1.0 : -1.0);
                    for (int i = 0; i < V; ++i) o[i] = load_logit(center, P->dtype, off + i) + sgn * r[i];
                    log_softmax(o, V, lp);
                    double l1 = 0.0, ce = 0.0, kl = 0.0;
                    for (int i = 0; i < V; ++i) {
                        const double pc = exp(lpc[i]), p = exp(lp[i]);
                        l1 += fabs(p - pc);
                        if (pc > 0.0) { ce -= pc * lp[i]; kl += pc * (lpc[i] - lp[i]); }
                    }
                    terms[(int64_t)v * N + n] = l1;
                    terms[(int64_t)(3 + v) * N + n] = ce;
                    if (v == 0) terms[6 * N + n] = kl;
                }
            }
        }
        free(o); free(lpc); free(lp); free(r);
    }
    if (!failed) {
        if (rows) memcpy(rows, terms, sizeof(double) * 7 * (size_t)N);
        const double* ce_lo = terms + 5 * N;
        double mx = -INFINITY;
        for (int64_t n = 0; n < N; ++n) if (alpha * ce_lo[n] > mx) mx = alpha * ce_lo[n];
        double den = 0.0;
        for (int64_t n = 0; n < N; ++n) den += exp(alpha * ce_lo[n] - mx);
        double dro = 0.0, centre = 0.0, upper = 0.0, lower = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            const double w = exp(alpha * ce_lo[n] - mx) / den;
            if (weights) weights[n] = w;
            dro += w * ce_lo[n];
            centre += lambda_v * terms[n] + lambda_p * terms[3 * N + n] + lambda_beta * terms[6 * N + n];
            upper  += lambda_v * terms[N + n] + lambda_p * terms[4 * N + n];
            lower  += lambda_v * terms[2 * N + n] + lambda_p * terms[5 * N + n];
        }
        if (N > 0) { centre /= (double)N; upper /= (double)N; lower /= (double)N; }
        if (losses) {
            losses[0] = centre; losses[1] = upper; losses[2] = lower; losses[3] = dro;
            losses[4] = centre + upper + lower + dro;
        }
    }
    free(terms);
    return failed ? -1 : 0;
}

/* ---- verification -------------------------------------------------------------------- */

/*
 * Residual distribution of one row: res_i = max(0, q_i - p_i) and its inclusive running
 * sum C_j in index order.  cdf must hold V doubles.  Returns R = C_{V-1}.
 */
double ciar_oracle_residual_cdf(const void* draft, const void* target, int64_t row,
                                const ciar_oracle_params* P, double* cdf)
{
    const int V = P->vocab;
    double* e  = (double*)malloc(sizeof(double) * (size_t)V);
    double* et = (double*)malloc(sizeof(double) * (size_t)V);
    if (!e || !et) { free(e); free(et); return NAN; }
    double m, mt;
    double S = row_exponentials(draft, P, row, e, &m);
    double Z = row_exponentials(target, P, row, et, &mt);
    double run = 0.0;
    for (int i = 0; i < V; ++i) {
        double res = et[i] / Z - e[i] / S;
        if (res < 0.0) res = 0.0;
        run += res;
        cdf[i] = run;
    }
    free(e); free(et);
    return run;
}

/*
 * Speculative verification of rows [0, N) in windows of K consecutive rows.
 *   accept[i]      = 1 iff ln(u_accept[i]) < min(0, ln q_x - ln p_x), x = ids[i]  (ln 0 = -inf: accept)
 *   row_id[i]      = -1 if accepted, else the residual sample:
 *                    the smallest j with C_j > u_resample[i] * R; if rounding leaves none, the largest j
 *                    with res_j > 0; if R == 0, the lowest-index argmax of q
 *   accept_len[w]  = number of leading accepted rows of window w = rows [wK, min((w+1)K, N))
 *   resampled[w]   = row_id of the first rejected row of the window, -1 if none
 * Diagnostics for the comparison's margin rule (any may be NULL):
 *   log_ratio[i]   = ln q_x - ln p_x
 *   res_margin[i]  = for rejected rows min(|C_id - T|, |C_{id-1} - T|) / R with T = u*R (C_{-1} = 0);
 *                    +inf for accepted rows and for R == 0
 */
int ciar_oracle_verify(const void* draft, const void* target, const int32_t* ids,
                       const float* u_accept, const float* u_resample, int64_t N,
                       const ciar_oracle_params* P,
                       uint8_t* accept, int32_t* row_id,
                       int32_t* accept_len, int32_t* resampled,
                       double* log_ratio, double* res_margin, int threads)
{
    const int V = P->vocab;
    const int64_t K = P->window;
    int failed = 0;
    if (threads < 1) threads = 1;
    uint8_t* acc_all = (uint8_t*)malloc((size_t)(N > 0 ? N : 1));
    int32_t* id_all  = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    if (!acc_all || !id_all) { free(acc_all); free(id_all); return -1; }

#pragma omp parallel num_threads(threads)
    {
        double* e  = (double*)malloc(sizeof(double) * (size_t)V);
        double* et = (double*)malloc(sizeof(double) * (size_t)V);
        if (!e || !et) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (int64_t row = 0; row < N; ++row) {
                double m, mt;
                double S = row_exponentials(draft, P, row, e, &m);
                double Z = row_exponentials(target, P, row, et, &mt);
                const int x = ids[row];
                const double cx = load_logit(draft, P->dtype, row * P->row_stride + x);
                const double tx = load_logit(target, P->dtype, row * P->row_stride + x);
                const double ell = (tx - mt - log(Z)) - (cx - m - log(S));
                const double lnu = log((double)u_accept[row]);        /* log(0) = -inf */
                const double bar = ell < 0.0 ? ell : 0.0;
                const int ok = lnu < bar;
                int id = -1;
                double margin = INFINITY;
                if (!ok) {
                    /* residual inverse-CDF draw, index order */
                    double R = 0.0;
                    for (int i = 0; i < V; ++i) {
                        double res = et[i] / Z - e[i] / S;
                        if (res > 0.0) R += res;
                    }
                    if (R > 0.0) {
                        const double T = (double)u_resample[row] * R;
                        double run = 0.0, prev = 0.0;
                        int last_positive = -1;
                        for (int i = 0; i < V; ++i) {
                            double res = et[i] / Z - e[i] / S;
                            if (res < 0.0) res = 0.0;
                            prev = run;
                            run += res;
                            if (res > 0.0) last_positive = i;
                            if (run > T) {
                                id = i;
                                double a = fabs(run - T), b = fabs(prev - T);
                                margin = (a < b ? a : b) / R;
                                break;
                            }
                        }
                        if (id < 0) { id = last_positive; margin = 0.0; }
                    } else {
                        id = lowest_argmax(et, V);
                    }
                }
                acc_all[row] = (uint8_t)ok;
                id_all[row] = id;
                if (log_ratio)  log_ratio[row] = ell;
                if (res_margin) res_margin[row] = margin;
            }
        }
        free(e); free(et);
    }

    if (!failed) {
        if (accept) memcpy(accept, acc_all, (size_t)N);
        if (row_id) memcpy(row_id, id_all, sizeof(int32_t) * (size_t)N);
        const int64_t W = (N + K - 1) / K;
        for (int64_t w = 0; w < W; ++w) {
            const int64_t lo = w * K, hi = (lo + K < N) ? lo + K : N;
            int64_t n = 0;
            while (lo + n < hi && acc_all[lo + n]) ++n;
            if (accept_len) accept_len[w] = (int32_t)n;
            if (resampled)  resampled[w] = (lo + n < hi) ? id_all[lo + n] : -1;
        }
    }
    free(acc_all); free(id_all);
    return failed ? -1 : 0;
}
