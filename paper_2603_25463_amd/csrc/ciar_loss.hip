// gfx950 kernels for the forward value of the Inter-DRO loss (Sec. 3.2.3: anchor, DRO and alignment
// equations): per-row terms, batch softmax weights and the batch reduction.
#include "ciar_device.h"

namespace ciar {
namespace {

// ---- Inter-DRO loss, forward (Sec. 3.2.3: anchor, DRO and alignment equations) -----------------------------

// e^((c + r) - (c* + r*)) for the token (c*, r*) that carries the row maximum of c + r, formed as
// (c - c*) + (r - r*): each difference is exact for tokens near the maximum and rounded relative to itself
// elsewhere, so c + r is never rounded to fp32.  That rounding, 6e-8 |c + r|, is a relative error of the same
// size in the token's probability, and for logits of magnitude ~30 it shows as ~1e-6 absolute in a cross-entropy
// (the difference of max + ln S and the p_cloud-weighted mean logit) and in an L1 distance.  The largest token
// contributes exactly 1 to S.  sign = +1 for c + r, -1 for c - r.
__device__ __forceinline__ float exp_rel(float c, float r, float cs, float rs, float sign)
{
    const float d = fmaf(sign, r - rs, c - cs);
    return __builtin_amdgcn_exp2f(fmaf(d, kLog2eLo, d * kLog2eHi));
}

// e^(x - m) for a row of plain logits.
__device__ __forceinline__ float exp_rel(float x, float m)
{
    const float d = x - m;
    return __builtin_amdgcn_exp2f(fmaf(d, kLog2eLo, d * kLog2eHi));
}

// Per-row terms of the loss.  One 1024-lane workgroup per row holds the centre, raw-radius and cloud rows as
// loaded (12 registers per vector) and makes three passes over them: the four maxima (of c, c + r, c - r and
// the cloud logits), the four partition sums together with sum p_cloud o for the cross-entropies, and the
// three L1 distances, which need all four normalisers.  With e = exp(o - max o):
//   CE(p_cloud, softmax(o)) = (max o + ln S_o) - (sum_i et_i o_i) / Z,
//   KL(p_cloud || p_mid)    = (sum_i et_i t_i) / Z - (max t + ln Z) + CE(p_cloud, p_mid).
// terms[k * N + row], k = 0..6: L1(mid), L1(up), L1(lo), CE(mid), CE(up), CE(lo), KL.
template <typename T, int NVEC>
__global__ __launch_bounds__(1024) void dro_row_kernel(const RowArgs A, float* __restrict__ terms)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec, THREADS = 1024, NW = 16;
    __shared__ double sm_d[NW * 7];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = A.V;
    const int last_vec = (V + EPV - 1) / EPV - 1;
    const bool rad = A.radius != nullptr;                          // uniform
    const float kap = (float)A.kappa, rmax = (float)A.rmax;
    const float r0 = (float)fmin(A.kappa, A.rmax);                 // the scalar radius

    const gbytes cb = (gbytes)(static_cast<const T*>(A.draft) + row * A.stride);
    const gbytes tb = (gbytes)(static_cast<const T*>(A.target) + row * A.stride);
    const gbytes rb = (gbytes)(static_cast<const T*>(rad ? A.radius : A.draft) + row * A.stride);
    u32x4 cw[NVEC], tw[NVEC], rw[NVEC];
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        const uint32_t off = (uint32_t)min(j * THREADS + tid, last_vec) * 16u;
        cw[j] = __builtin_nontemporal_load((gvec)(cb + off));     // every row is used once: stream past the caches
        tw[j] = __builtin_nontemporal_load((gvec)(tb + off));
        if (rad) rw[j] = __builtin_nontemporal_load((gvec)(rb + off));
    }
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        const int base = (j * THREADS + tid) * EPV;
        E::mask_tail(cw[j], base, V);
        E::mask_tail(tw[j], base, V);
        if (rad) E::zero_tail(rw[j], base, V);
    }
    // The radii are formed once (Softplus costs about as much as the rest of a pass) and kept as floats where
    // the registers allow: up to 32 tokens per lane.  Beyond that they are recomputed in every pass.
    constexpr bool CACHE_R = NVEC * EPV <= 32;
    float rc[CACHE_R ? NVEC * EPV : 1];
    if constexpr (CACHE_R) {
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            float rv[EPV];
            if (rad) E::unpack(rw[j], rv);
#pragma unroll
            for (int k = 0; k < EPV; ++k) rc[j * EPV + k] = rad ? radius_r(rv[k], kap, rmax) : r0;
        }
    }
    // element k of vector j: centre logit, radius, cloud logit
    auto element = [&](int j, int k, float& c, float& r, float& t) {
        float cv[EPV], tv[EPV], rv[EPV];
        E::unpack(cw[j], cv);
        E::unpack(tw[j], tv);
        c = cv[k]; t = tv[k];
        if constexpr (CACHE_R) {
            r = rc[j * EPV + k];
        } else {
            r = r0;
            if (rad) { E::unpack(rw[j], rv); r = radius_r(rv[k], kap, rmax); }
        }
    };
    // The three passes recompute the radius and the sums c +- r from the rows as loaded.  Passing the row
    // registers through an empty asm before each pass keeps the optimiser from carrying every per-token
    // value of one pass over to the next (which would triple the registers the rows themselves need).
    auto fresh = [&]() {
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            asm volatile("" : "+v"(cw[j]), "+v"(tw[j]));
            if (!CACHE_R && rad) asm volatile("" : "+v"(rw[j]));
        }
    };
    // pass 1: the four maxima; for c + r and c - r also the (c, r) of the token that carries the maximum
    float mc = -INFINITY, mt = -INFINITY;
    float su = -INFINITY, cu = 0.f, ru = 0.f;                      // max of c + r and its token
    float sl = -INFINITY, cl = 0.f, rl = 0.f;                      // max of c - r and its token
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float c, r, t;
            element(j, k, c, r, t);
            mc = fmaxf(mc, c); mt = fmaxf(mt, t);
            const float s1 = c + r, s2 = c - r;
            if (s1 > su) { su = s1; cu = c; ru = r; }
            if (s2 > sl) { sl = s2; cl = c; rl = r; }
        }
    }
    {
        // wave: the lowest lane that holds the wave's maximum hands over its token
        auto wave_argmax = [&](float& sv, float& cv, float& rv) {
            const float w = wave_max(sv);
            const unsigned long long b = __ballot(sv == w);
            const int src = b ? __ffsll((long long)b) - 1 : 0;
            cv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cv), src));
            rv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(rv), src));
            sv = w;
        };
        mc = wave_max(mc); mt = wave_max(mt);
        wave_argmax(su, cu, ru);
        wave_argmax(sl, cl, rl);
        float* slot = reinterpret_cast<float*>(sm_d);              // 8 floats per wave (sm_d holds 7 doubles per wave)
        if (lane == 0) {
            float* q = slot + wave * 8;
            q[0] = mc; q[1] = mt; q[2] = su; q[3] = cu; q[4] = ru; q[5] = sl; q[6] = cl; q[7] = rl;
        }
        __syncthreads();
        // every wave combines the sixteen waves' results across its lanes: lane l takes wave l & 15 (the copies in
        // the upper lanes change no maximum, and the lowest lane that holds a maximum is the lowest wave)
        {
            const float* q = slot + (lane & 15) * 8;
            mc = wave_max(q[0]); mt = wave_max(q[1]);
            su = q[2]; cu = q[3]; ru = q[4];
            sl = q[5]; cl = q[6]; rl = q[7];
            wave_argmax(su, cu, ru);
            wave_argmax(sl, cl, rl);
        }
        __syncthreads();                                           // sm_d is reused below
    }
    // a row without a live token: any finite reference will do (every exponential is 0)
    if (mc == -INFINITY) mc = 0.f;
    if (mt == -INFINITY) mt = 0.f;
    // the references are the same in every lane: keep them in scalar registers
    auto uniform = [](float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); };
    mc = uniform(mc); mt = uniform(mt);
    cu = uniform(cu); ru = uniform(ru); cl = uniform(cl); rl = uniform(rl);
    const double mu = (double)cu + (double)ru, ml = (double)cl - (double)rl;   // the two maxima, exact

    // pass 2: partition sums and the p_cloud-weighted sums of c, r and the cloud logits
    fresh();
    double acc[7] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};          // S_mid, S_up, S_lo, Z, sum et c, sum et r, sum et t
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float c, r, t;
            element(j, k, c, r, t);
            const float et = exp_rel(t, mt);
            acc[0] += (double)exp_rel(c, mc);
            acc[1] += (double)exp_rel(c, r, cu, ru, 1.f);
            acc[2] += (double)exp_rel(c, r, cl, rl, -1.f);
            acc[3] += (double)et;
            if (et > 0.f) {                                        // a token the cloud rules out weighs nothing
                acc[4] = fma((double)et, (double)c, acc[4]);
                acc[5] = fma((double)et, (double)r, acc[5]);
                acc[6] = fma((double)et, (double)t, acc[6]);
            }
            if (k & 1) __builtin_amdgcn_sched_barrier(0);          // two tokens at a time: bounded working set
        }
    }
#pragma unroll
    for (int i = 0; i < 7; ++i) acc[i] = wave_sum(acc[i]);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < 7; ++i) sm_d[wave * 7 + i] = acc[i];
    }
    __syncthreads();
    // the sixteen waves' sums, one per lane of the first DPP row, added across that row in every wave
    double tot[7];
#pragma unroll
    for (int i = 0; i < 7; ++i) tot[i] = row16_sum(lane < NW ? sm_d[lane * 7 + i] : 0.0);
    __syncthreads();                                               // sm_d is reused below

    // pass 3: L1 distances to p_cloud
    const float is0 = (float)(1.0 / tot[0]), is1 = (float)(1.0 / tot[1]), is2 = (float)(1.0 / tot[2]),
                iz = (float)(1.0 / tot[3]);
    double l1[3] = {0.0, 0.0, 0.0};
    fresh();
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float c, r, t;
            element(j, k, c, r, t);
            const float pc = exp_rel(t, mt) * iz;
            l1[0] += (double)fabsf(exp_rel(c, mc) * is0 - pc);
            l1[1] += (double)fabsf(exp_rel(c, r, cu, ru, 1.f) * is1 - pc);
            l1[2] += (double)fabsf(exp_rel(c, r, cl, rl, -1.f) * is2 - pc);
            if (k & 1) __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int i = 0; i < 3; ++i) l1[i] = wave_sum(l1[i]);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < 3; ++i) sm_d[wave * 7 + i] = l1[i];
    }
    __syncthreads();
    if (wave == 0) {
        double L[3];
#pragma unroll
        for (int i = 0; i < 3; ++i) L[i] = row16_sum(lane < NW ? sm_d[lane * 7 + i] : 0.0);
        // the four logarithms side by side: lane i takes ln tot[i]
        const double mine = lane == 0 ? tot[0] : lane == 1 ? tot[1] : lane == 2 ? tot[2] : tot[3];
        const double lg = log(mine);
        auto from_lane = [&](int src) {
            return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(lg), src),
                                    __builtin_amdgcn_readlane(__double2loint(lg), src));
        };
        const double ln_s0 = from_lane(0), ln_s1 = from_lane(1), ln_s2 = from_lane(2), ln_z = from_lane(3);
        if (lane != 0) return;
        const double Z = tot[3];
        const double pc_c = tot[4] / Z, pc_r = tot[5] / Z, pc_t = tot[6] / Z;
        const double ce_mid = ((double)mc + ln_s0) - pc_c;
        const double ce_up = (mu + ln_s1) - (pc_c + pc_r);
        const double ce_lo = (ml + ln_s2) - (pc_c - pc_r);
        const double kl = pc_t - ((double)mt + ln_z) + ce_mid;
        const int64_t N = A.N;
        terms[0 * N + row] = (float)L[0]; terms[1 * N + row] = (float)L[1]; terms[2 * N + row] = (float)L[2];
        terms[3 * N + row] = (float)ce_mid; terms[4 * N + row] = (float)ce_up; terms[5 * N + row] = (float)ce_lo;
        terms[6 * N + row] = (float)kl;
    }
}

// The same terms for a handful of tokens (V <= kTinyVocab): one thread per row, fp64 throughout.  With so few
// tokens a cross-entropy can be close to zero, where the difference (n ln2 + ln S) - sum p_cloud o formed from
// fp32 exponentials keeps only ~5e-7 absolute.
template <typename T>
__global__ __launch_bounds__(256) void dro_row_tiny_kernel(const RowArgs A, float* __restrict__ terms)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= A.N) return;
    const int V = A.V;
    const T* c = static_cast<const T*>(A.draft) + row * A.stride;
    const T* t = static_cast<const T*>(A.target) + row * A.stride;
    const T* rr = A.radius ? static_cast<const T*>(A.radius) + row * A.stride : nullptr;
    const double r0 = fmin(A.kappa, A.rmax);
    auto radius = [&](int i) { return rr ? radius_of((double)load_logit(rr, i), A.kappa, A.rmax) : r0; };
    double m[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    for (int i = 0; i < V; ++i) {
        const double ci = (double)load_logit(c, i), ri = radius(i);
        m[0] = fmax(m[0], ci); m[1] = fmax(m[1], ci + ri); m[2] = fmax(m[2], ci - ri);
        m[3] = fmax(m[3], (double)load_logit(t, i));
    }
    double S[4] = {0.0, 0.0, 0.0, 0.0}, Tc = 0.0, Tr = 0.0, Tt = 0.0;
    for (int i = 0; i < V; ++i) {
        const double ci = (double)load_logit(c, i), ri = radius(i), ti = (double)load_logit(t, i);
        const double et = exp(ti - m[3]);
        S[0] += exp(ci - m[0]); S[1] += exp(ci + ri - m[1]); S[2] += exp(ci - ri - m[2]); S[3] += et;
        if (et > 0.0) { Tc = fma(et, ci, Tc); Tr = fma(et, ri, Tr); Tt = fma(et, ti, Tt); }
    }
    double L[3] = {0.0, 0.0, 0.0};
    for (int i = 0; i < V; ++i) {
        const double ci = (double)load_logit(c, i), ri = radius(i);
        const double pc = exp((double)load_logit(t, i) - m[3]) / S[3];
        L[0] += fabs(exp(ci - m[0]) / S[0] - pc);
        L[1] += fabs(exp(ci + ri - m[1]) / S[1] - pc);
        L[2] += fabs(exp(ci - ri - m[2]) / S[2] - pc);
    }
    // sum_i pc_i (lnZ_o - o_i) with lnZ_o - o_i >= 0 term by term would need another pass; the difference
    // below is exact enough in fp64
    const double pc_c = Tc / S[3], pc_r = Tr / S[3], pc_t = Tt / S[3];
    const double ce_mid = (m[0] + log(S[0])) - pc_c;
    const double ce_up = (m[1] + log(S[1])) - (pc_c + pc_r);
    const double ce_lo = (m[2] + log(S[2])) - (pc_c - pc_r);
    const double kl = pc_t - (m[3] + log(S[3])) + ce_mid;
    const int64_t N = A.N;
    terms[0 * N + row] = (float)L[0]; terms[1 * N + row] = (float)L[1]; terms[2 * N + row] = (float)L[2];
    terms[3 * N + row] = (float)ce_mid; terms[4 * N + row] = (float)ce_up; terms[5 * N + row] = (float)ce_lo;
    terms[6 * N + row] = (float)kl;
}

// Batch stage: w_n = softmax_n(alpha CE_n(p_lo)), DRO = sum w CE(p_lo), batch means of the anchor and alignment
// terms.  One workgroup; losses = { centre, upper, lower, DRO, total }.
__global__ __launch_bounds__(1024) void dro_batch_kernel(const float* __restrict__ terms, int64_t N, double lambda_v,
                                                         double lambda_p, double lambda_beta, double alpha,
                                                         float* __restrict__ weights, float* __restrict__ losses)
{
    constexpr int NW = 16;
    __shared__ double sm[NW * 4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* ce_lo = terms + 5 * N;
    auto block_sum = [&](double v, int slot) -> double {
        v = wave_sum(v);
        if (lane == 0) sm[wave * 4 + slot] = v;
        __syncthreads();
        double t = 0.0;
        for (int w = 0; w < NW; ++w) t += sm[w * 4 + slot];
        __syncthreads();
        return t;
    };
    float mxf = -INFINITY;
    double c = 0.0, u = 0.0, l = 0.0;
    for (int64_t n = tid; n < N; n += 1024) {
        mxf = fmaxf(mxf, (float)(alpha * (double)ce_lo[n]));
        c += lambda_v * terms[n] + lambda_p * terms[3 * N + n] + lambda_beta * terms[6 * N + n];
        u += lambda_v * terms[N + n] + lambda_p * terms[4 * N + n];
        l += lambda_v * terms[2 * N + n] + lambda_p * terms[5 * N + n];
    }
    mxf = wave_max(mxf);
    if (lane == 0) sm[wave * 4] = (double)mxf;
    __syncthreads();
    double mx = sm[0];
    for (int w = 1; w < NW; ++w) mx = fmax(mx, sm[w * 4]);
    __syncthreads();
    c = block_sum(c, 0); u = block_sum(u, 1); l = block_sum(l, 2);
    double den = 0.0;
    for (int64_t n = tid; n < N; n += 1024) den += exp(alpha * (double)ce_lo[n] - mx);
    den = block_sum(den, 3);
    double dro = 0.0;
    for (int64_t n = tid; n < N; n += 1024) {
        const double w = exp(alpha * (double)ce_lo[n] - mx) / den;
        if (weights) weights[n] = (float)w;
        dro = fma(w, (double)ce_lo[n], dro);
    }
    dro = block_sum(dro, 0);
    if (tid == 0 && losses) {
        const double Nd = (double)N;
        losses[0] = (float)(c / Nd); losses[1] = (float)(u / Nd); losses[2] = (float)(l / Nd); losses[3] = (float)dro;
        losses[4] = (float)(c / Nd + u / Nd + l / Nd + dro);
    }
}

}  // namespace

hipError_t launch_dro(int dtype, const RowArgs& args, float* terms, double lambda_v, double lambda_p,
                      double lambda_beta, double alpha, float* weights, float* losses, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const int epv = dtype == 0 ? 4 : 8;
    const int vecs = (args.V + epv - 1) / epv;
    const dim3 grid((unsigned)args.N), block(1024);
#define CIAR_DRO_LAUNCH(NV)                                                                             \
    do {                                                                                                \
        if (dtype == 0) hipLaunchKernelGGL((dro_row_kernel<float, NV>), grid, block, 0, stream, args, terms);   \
        else hipLaunchKernelGGL((dro_row_kernel<bf16_t, NV>), grid, block, 0, stream, args, terms);              \
    } while (0)
    if (args.V <= kTinyVocab) {
        const dim3 tgrid((unsigned)((args.N + 255) / 256)), tblock(256);
        if (dtype == 0) hipLaunchKernelGGL(dro_row_tiny_kernel<float>, tgrid, tblock, 0, stream, args, terms);
        else hipLaunchKernelGGL(dro_row_tiny_kernel<bf16_t>, tgrid, tblock, 0, stream, args, terms);
    } else if (vecs <= 1024) CIAR_DRO_LAUNCH(1);
    else if (vecs <= 2048) CIAR_DRO_LAUNCH(2);
    else if (vecs <= 4096) CIAR_DRO_LAUNCH(4);
    else if (vecs <= 8192) CIAR_DRO_LAUNCH(8);
    else return hipErrorInvalidValue;
#undef CIAR_DRO_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || (!weights && !losses)) return e;
    hipLaunchKernelGGL(dro_batch_kernel, dim3(1), dim3(1024), 0, stream, terms, args.N, lambda_v, lambda_p,
                       lambda_beta, alpha, weights, losses);
    return hipGetLastError();
}

}  // namespace ciar
