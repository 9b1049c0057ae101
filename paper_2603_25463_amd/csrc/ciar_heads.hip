// gfx950 kernels for several Interval Heads (Sec. 4, ablation on the Inter-Head): the Ensemble sweep that
// averages the heads' widths token by token, and the Voting majority.
#include "ciar_device.h"

#include <mutex>
#include <type_traits>

namespace ciar {
namespace {

// ---- several heads (Sec. 4, ablation on the Inter-Head): Ensemble and Voting ------------------------------

constexpr int kMaxHeads = 8;

// Ensemble: the heads' curves are averaged token by token, so the widths of all heads of a token have to
// meet: a second sweep over the H rows of a position, after the streaming kernel has left every head's
// RowStats (partition sum, reference, interval sums -> that head's caps).  One workgroup per position;
// per token and head the same arithmetic as the streaming kernel's interval pass.
//   D_i = sum_h delta_{h,i},  Omega = sum_i D_i / H,  Sigma^2 = sum_i D_i^2 / (H^2 V) - (Omega / V)^2.
// WIDE (calls with a wide radius, see wide_radius): also C_i = sum_h (1 - width_{h,i}); where every mean width is
// above 1/2 and no head has an active cap, D_i = H - C_i, and Omega and Sigma are taken from the sums of C_i,
// which resolve a spread that the widths, all rounding to 1, no longer show.
template <typename T, bool WIDE>
__global__ __launch_bounds__(256) void ensemble_kernel(const RowArgs A, const int H, const int64_t head_stride)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec;
    __shared__ FuseRow sm_fr[kMaxHeads];
    __shared__ float sm_n[kMaxHeads], sm_invS[kMaxHeads];
    __shared__ double sm_cw[kMaxHeads], sm_cl[kMaxHeads], sm_S[kMaxHeads], sm_al[kMaxHeads], sm_au[kMaxHeads];
    __shared__ double sm_red[5][4];
    __shared__ float sm_pm[4];
    __shared__ int sm_pi[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = A.V;
    const bool rad = A.radius != nullptr;
    const bool need_argmax = A.ids == nullptr && (A.p_lo || A.p_mid || A.p_hi);
    bool flat_h = true;                                            // this lane's head: a flat row (see below)

    if (tid < H) {
        const RowStats st = A.stats[(int64_t)tid * A.N + row];
        flat_h = (double)exp2_ref(st.mc, st.n == -INFINITY ? 0.f : st.n) * (double)V <= 2.0 * st.S;
        const RowScore rs = finish_score(st.q, st.S, st.mode, A, st.kl, st.kw);
        const double Bc = (rad ? 1.0 : A.b) / st.S, Wc = (rad ? 1.0 : A.a - A.b) / st.S;
        sm_fr[tid] = fuse_row(st.S, A.a, A.b);
        sm_n[tid] = st.n;
        sm_cw[tid] = rs.alpha_u * Wc;
        sm_cl[tid] = (rs.alpha_u - rs.alpha_l) * Bc;
        sm_invS[tid] = (float)(1.0 / st.S);
        sm_S[tid] = st.S; sm_al[tid] = rs.alpha_l; sm_au[tid] = rs.alpha_u;
    }
    // Token arithmetic in fp64 ("precise") for rows of a handful of tokens and for rows that are flat in every
    // head (largest probability <= 2 / V): there the widths can agree to 1e-4 and better while their fp32 errors
    // (~1e-7 each, uncorrelated when the radii differ from token to token) do not, and Omega ~ V multiplies what
    // is left of the spread.
    const bool precise = __syncthreads_and(flat_h ? 1 : 0) != 0 || V <= 64;   // uniform; also the barrier
    // no head with an active cap (delta = alpha_u w + (alpha_u - alpha_l) p^l loses its second term): uniform
    const bool no_lower = __syncthreads_and(tid < H ? (sm_cl[tid] == 0.0 ? 1 : 0) : 1) != 0;

    const RadiusMode rm = radius_mode(A);
    const int nvec = (V + EPV - 1) / EPV;
    // One head's share of a token: its width after the head's caps (added to d) and, WIDE, its complement (to c).
    auto head_token = [&](int h, float cval, float rval, const FuseRow& fr, double& d, double& c) {
        const float e = exp2_ref(cval, sm_n[h]);
        float gl, gw;
        if constexpr (WIDE) {
            float ec;
            if (rad) fuse_token_rad_wide(e, rval, fr, rm, gl, gw, ec);
            else fuse_token_wide(e, fr, gl, gw, ec);
            c += (double)ec;
        } else {
            if (rad) fuse_token_rad(e, rval, fr, rm, gl, gw);
            else fuse_token(e, fr, gl, gw);
        }
        d = fma(sm_cw[h], (double)gw, fma(sm_cl[h], (double)gl, d));
        return e;
    };
    // The same in fp64 from the fp32 e (rows of a handful of tokens).
    auto head_token_tiny = [&](int h, float cval, float rval, double& d, double& c) {
        // A handful of tokens: e as the streaming kernel summed it into S, so that 1 - x stays accurate as x -> 1.
        // A flat row: the fp64 exponential (every x is tiny; the fp32 one would leave 6e-8 of each width behind,
        // uncorrelated from token to token, where the widths themselves agree to 1e-6).
        const double ed = V <= 64 ? (double)exp2_ref(cval, sm_n[h]) : exp((double)cval - (double)sm_n[h] * kLn2);
        const double x = ed / sm_S[h], omx = fmax(0.0, sm_S[h] - ed) / sm_S[h];
        double a = A.a, b = A.b;
        if (rad) {
            const double rr = radius_of((double)rval, A.kappa, A.rmax);
            a = exp(rr); b = exp(-rr);
        }
        const double du = 1.0 + (a - 1.0) * x, dl = b + (1.0 - b) * omx;
        d += sm_au[h] * a * x / du - sm_al[h] * b * x / dl;
        if constexpr (WIDE) c += (1.0 - 2.0 * (1.0 - b) * x * omx) / (du * dl);
        return x;
    };
    // The sums over the tokens are taken about D and C of the row's first token (every lane forms the same two
    // numbers): the spread of a row whose widths all agree is then 0 instead of the rounding noise that the
    // difference of two large moments leaves.
    double KD = 0.0, KC = 0.0;
    auto first_token = [&](bool in_fp64) {
        KD = 0.0; KC = 0.0;
        for (int h = 0; h < H; ++h) {
            const T* crow = static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride;
            const T* rrow = static_cast<const T*>(rad ? A.radius : A.draft) + (int64_t)h * head_stride + row * A.stride;
            const float c0 = load_logit(crow, 0), r0 = load_logit(rrow, 0);
            if (in_fp64) head_token_tiny(h, c0, r0, KD, KC);
            else head_token(h, c0, r0, sm_fr[h], KD, KC);
        }
    };
    first_token(precise);
    double s1 = 0.0, s2 = 0.0;                                     // sum (D_i - KD), sum (D_i - KD)^2
    double c1 = 0.0, c2 = 0.0, cbig = 0.0;                         // WIDE: sum (C_i - KC), its square, max C_i
    float best = -INFINITY;
    int best_i = INT_MAX;
    auto precise_sweep = [&]() {
        s1 = 0.0; s2 = 0.0; c1 = 0.0; c2 = 0.0; cbig = 0.0;
        best = -INFINITY; best_i = INT_MAX;
        for (int v = tid; v < nvec; v += 256) {
            double D[EPV], C[EPV];
            float pm[EPV];
#pragma unroll
            for (int k = 0; k < EPV; ++k) { D[k] = 0.0; C[k] = 0.0; pm[k] = 0.f; }
            for (int h = 0; h < H; ++h) {
                const gvec c = (gvec)(gbytes)(static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride);
                const gvec r = (gvec)(gbytes)(static_cast<const T*>(rad ? A.radius : A.draft) +
                                              (int64_t)h * head_stride + row * A.stride);
                const u32x4 cw4 = c[v], rw4 = r[v];
                float cv[EPV], rv[EPV];
                E::unpack(cw4, cv);
                E::unpack(rw4, rv);
                for (int k = 0; k < EPV; ++k) {
                    if (v * EPV + k < V) pm[k] += (float)head_token_tiny(h, cv[k], rv[k], D[k], C[k]);
                }
            }
            for (int k = 0; k < EPV; ++k) {
                const int tok = v * EPV + k;
                if (tok < V) {
                    const double d = D[k] - KD;
                    s1 += d;
                    s2 = fma(d, d, s2);
                    if constexpr (WIDE) {
                        const double c = C[k] - KC;
                        c1 += c; c2 = fma(c, c, c2); cbig = fmax(cbig, C[k]);
                    }
                }
                if (need_argmax && tok < V && pm[k] > best) { best = pm[k]; best_i = tok; }
            }
        }
    };
    if (precise) precise_sweep();
    // The sweep proper, specialised on what is uniform over the launch or the row: MODE bit 0 = tensor radius,
    // bit 1 = unit radius scale (see radius_am1), bit 2 = no head has an active cap (p^l is not needed).
    // Two 16-byte vectors of a head in flight per lane (fp32; one for bf16): more of them cost registers and
    // with them a wave per SIMD, which measured slower (four: +4 %, eight: +70 %).
    constexpr int UB = EPV >= 8 ? 1 : 8 / EPV;
    auto sweep = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;
        constexpr bool RADc = (MODE & 1) != 0, UNITc = (MODE & 2) != 0, NOLOW = (MODE & 4) != 0;
        for (int v0 = tid; v0 < nvec; v0 += 256 * UB) {
            double D[UB][EPV];                                     // fp64 across heads
            double C[WIDE ? UB : 1][EPV];
            float pm[UB][EPV];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    D[u][k] = 0.0; pm[u][k] = 0.f;
                    if constexpr (WIDE) C[u][k] = 0.0;
                }
            }
            for (int h = 0; h < H; ++h) {
                const gvec c = (gvec)(gbytes)(static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride);
                const gvec r = (gvec)(gbytes)(static_cast<const T*>(RADc ? A.radius : A.draft) +
                                              (int64_t)h * head_stride + row * A.stride);
                u32x4 cw4[UB], rw4[UB];
#pragma unroll
                for (int u = 0; u < UB; ++u) cw4[u] = c[min(v0 + u * 256, nvec - 1)];
                if constexpr (RADc) {
#pragma unroll
                    for (int u = 0; u < UB; ++u) rw4[u] = r[min(v0 + u * 256, nvec - 1)];
                }
                const FuseRow fr = sm_fr[h];
                const float invS = sm_invS[h], nh = sm_n[h];
                const double cw = sm_cw[h], cl = sm_cl[h];
                auto token = [&](float cval, float rval, double& d, double& cc, float& p) {
                    const float e = exp2_ref(cval, nh);
                    float gl, gw;
                    if constexpr (WIDE) {
                        float ec;
                        if constexpr (RADc) fuse_token_rad_wide<UNITc>(e, rval, fr, rm.kappa, rm.rmax, rm.am1_max, gl, gw, ec);
                        else fuse_token_wide(e, fr, gl, gw, ec);
                        cc += (double)ec;
                    } else {
                        if constexpr (RADc) fuse_token_rad<UNITc>(e, rval, fr, rm.kappa, rm.rmax, rm.am1_max, gl, gw);
                        else fuse_token(e, fr, gl, gw);
                    }
                    if constexpr (NOLOW) d = fma(cw, (double)gw, d);
                    else d = fma(cw, (double)gw, fma(cl, (double)gl, d));
                    p = fmaf(e, invS, p);
                };
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    const int tok0 = (v0 + u * 256) * EPV;         // >= V for vectors past the row's end
                    float cv[EPV], rv[EPV];
                    E::unpack(cw4[u], cv);
                    if constexpr (RADc) E::unpack(rw4[u], rv);
                    if (tok0 + EPV <= V) {                         // a whole vector of tokens: no per-token test
#pragma unroll
                        for (int k = 0; k < EPV; ++k) token(cv[k], RADc ? rv[k] : 0.f, D[u][k], C[WIDE ? u : 0][k], pm[u][k]);
                    } else {
#pragma unroll
                        for (int k = 0; k < EPV; ++k) {
                            if (tok0 + k < V) token(cv[k], RADc ? rv[k] : 0.f, D[u][k], C[WIDE ? u : 0][k], pm[u][k]);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    const int tok = (v0 + u * 256) * EPV + k;
                    if (tok < V) {
                        const double d = D[u][k] - KD;
                        s1 += d;
                        s2 = fma(d, d, s2);
                        if constexpr (WIDE) {
                            const double c = C[u][k] - KC;
                            c1 += c; c2 = fma(c, c, c2); cbig = fmax(cbig, C[u][k]);
                        }
                    }
                    if (need_argmax && tok < V && pm[u][k] > best) { best = pm[u][k]; best_i = tok; }
                }
            }
        }
    };
    if (!precise) {
        const int mode = (rad ? 1 : 0) | (rad && rm.unit ? 2 : 0) | (no_lower ? 4 : 0);
        switch (mode) {
        case 0: sweep(std::integral_constant<int, 0>{}); break;
        case 1: sweep(std::integral_constant<int, 1>{}); break;
        case 3: sweep(std::integral_constant<int, 3>{}); break;
        case 4: sweep(std::integral_constant<int, 4>{}); break;
        case 5: sweep(std::integral_constant<int, 5>{}); break;
        default: sweep(std::integral_constant<int, 7>{}); break;
        }
    }
    auto reduce = [&]() {
        s1 = wave_sum(s1);
        s2 = wave_sum(s2);
        if (lane == 0) { sm_red[0][wave] = s1; sm_red[1][wave] = s2; }
        if constexpr (WIDE) {
            c1 = wave_sum(c1);
            c2 = wave_sum(c2);
            cbig = (double)wave_max((float)cbig);
            if (lane == 0) { sm_red[2][wave] = c1; sm_red[3][wave] = c2; sm_red[4][wave] = cbig; }
        }
        if (need_argmax) {
            // each lane walked its tokens in ascending order, so it holds its lowest index of its maximum
            const float wm = wave_max(best);
            const int wi = wave_min_i(best == wm ? best_i : INT_MAX);
            if (lane == 0) { sm_pm[wave] = wm; sm_pi[wave] = wi; }
        }
        __syncthreads();
    };
    reduce();
    if (!precise) {
        // A row whose averaged widths agree to better than a hundredth of their mean although it is not flat in the
        // centre logits (heads whose widths crowd against 1 averaged with heads whose widths are next to nothing: every
        // D_i is about the same number): the ~1e-7 that fp32 token arithmetic leaves in each width is then no longer
        // small against the spread, and Omega multiplies what it does to Sigma (a seeded random case with a
        // tensor radius of scale 17: score off by 2e-5 of itself).  Such rows -- rare -- are swept again in fp64.
        // Every lane takes the same decision from the same numbers.
        const double t1 = (sm_red[0][0] + sm_red[0][1]) + (sm_red[0][2] + sm_red[0][3]);
        const double t2 = (sm_red[1][0] + sm_red[1][1]) + (sm_red[1][2] + sm_red[1][3]);
        const double Vd = (double)V, mean = (t1 + Vd * KD) / Vd, varD = fmax(0.0, t2 - t1 * t1 / Vd) / Vd;
        bool tight = varD < 1e-4 * mean * mean;
        if constexpr (WIDE) {
            // (not where the complement sums are read: they resolve exactly this case on their own)
            const double ub = fmax(fmax(sm_red[4][0], sm_red[4][1]), fmax(sm_red[4][2], sm_red[4][3]));
            bool plain = ub < kComplementBelow * (double)H;
            for (int h = 0; h < H; ++h) plain = plain && sm_al[h] == 1.0 && sm_au[h] == 1.0;
            tight = tight && !plain;
        }
        if (tight) {
            __syncthreads();                                       // sm_red is read by every lane above
            first_token(true);
            precise_sweep();
            reduce();
        }
    }
    if (tid == 0) {
        const double t1 = (sm_red[0][0] + sm_red[0][1]) + (sm_red[0][2] + sm_red[0][3]);
        const double t2 = (sm_red[1][0] + sm_red[1][1]) + (sm_red[1][2] + sm_red[1][3]);
        const double Hd = (double)H, Vd = (double)V;
        // t1 = sum (D_i - KD), t2 = sum (D_i - KD)^2
        double omega = (t1 + Vd * KD) / Hd;
        double var = fmax(0.0, t2 - t1 * t1 / Vd) / (Hd * Hd * Vd);
        if constexpr (WIDE) {
            const double u1 = (sm_red[2][0] + sm_red[2][1]) + (sm_red[2][2] + sm_red[2][3]);
            const double u2 = (sm_red[3][0] + sm_red[3][1]) + (sm_red[3][2] + sm_red[3][3]);
            const double ub = fmax(fmax(sm_red[4][0], sm_red[4][1]), fmax(sm_red[4][2], sm_red[4][3]));
            bool plain = ub < kComplementBelow * Hd;               // every mean width above 1/2
            for (int h = 0; h < H; ++h) plain = plain && sm_al[h] == 1.0 && sm_au[h] == 1.0;
            if (plain) {
                omega = Vd - (u1 + Vd * KC) / Hd;
                var = fmax(0.0, u2 - u1 * u1 / Vd) / (Hd * Hd * Vd);
            }
        }
        const double sigma = sqrt(var), score = omega * sigma;
        if (A.omega) A.omega[row] = (float)omega;
        if (A.sigma) A.sigma[row] = (float)sigma;
        if (A.score) A.score[row] = (float)score;
        if (A.flags) A.flags[row] = (uint8_t)(score > A.tau);
        if (A.p_lo || A.p_mid || A.p_hi) {
            int xid;
            if (A.ids) {
                xid = A.ids[row];
                xid = xid < 0 ? 0 : (xid >= V ? V - 1 : xid);
            } else {
                const float rm = fmaxf(fmaxf(sm_pm[0], sm_pm[1]), fmaxf(sm_pm[2], sm_pm[3]));
                xid = INT_MAX;
                for (int w = 0; w < 4; ++w) if (sm_pm[w] == rm && sm_pi[w] < xid) xid = sm_pi[w];
                if (xid == INT_MAX) xid = 0;
            }
            double lo = 0.0, mid = 0.0, hi = 0.0;
            for (int h = 0; h < H; ++h) {
                const T* crow = static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride;
                const double ex = (double)exp2_ref(load_logit(crow, xid), sm_n[h]);
                const double x = ex / sm_S[h], omx = fmax(0.0, sm_S[h] - ex) / sm_S[h];
                double a = A.a, b = A.b;
                if (rad) {
                    const T* rrow = static_cast<const T*>(A.radius) + (int64_t)h * head_stride + row * A.stride;
                    const double r = radius_of((double)load_logit(rrow, xid), A.kappa, A.rmax);
                    a = exp(r); b = exp(-r);
                }
                mid += x;
                lo += sm_al[h] * b * x / (b + (1.0 - b) * omx);
                hi += sm_au[h] * a * x / (1.0 + (a - 1.0) * x);
            }
            if (A.p_lo) A.p_lo[row] = (float)(lo / Hd);
            if (A.p_mid) A.p_mid[row] = (float)(mid / Hd);
            if (A.p_hi) A.p_hi[row] = (float)(hi / Hd);
        }
    }
}

// Values that are the same in every lane of a wave, moved to scalar registers.
__device__ __forceinline__ float uniform_f(float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); }
__device__ __forceinline__ double uniform_d(double v)
{
    const long long b = __double_as_longlong(v);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ FuseRow uniform_fr(FuseRow r)
{
    r.cu = uniform_f(r.cu); r.nih = uniform_f(r.nih); r.nil = uniform_f(r.nil); r.b = uniform_f(r.b); r.omb = uniform_f(r.omb);
    return r;
}
// 2^k as a double for an integer-valued float k of either sign (clamped to what a double holds)
__device__ __forceinline__ double pow2_any(float k) { return ldexp(1.0, (int)fminf(fmaxf(k, -1000.f), 1000.f)); }

// Ensemble in one sweep, for up to kFusedHeads heads with a scalar radius whose rows fit a 512-lane workgroup
// (32 elements of a row per lane): every head's row of a position is read from memory once.  A workgroup takes one
// position at a time and two workgroups share a compute unit, one waiting for its rows while the other computes.
// The exponentials of two heads stay in registers; a third head's go through LDS (64 KiB per workgroup, each lane
// writing and reading its own slots), because three rows and the working set do not fit 128 registers.
// Per position:
//   1. as each head's row arrives: per-wave maximum, e_i = 2^(c_i log2e - n_w) in place of the logits, S_w;
//      -- barrier: the waves exchange (max, n_w, S_w) of every head --
//   2. every wave forms each head's S and reference.  Heads whose largest probability is below the host's bound
//      have inactive caps; if some head may have an active cap, every head's sums of p^l and of the widths are
//      taken first (one more exchange), which gives the caps.
//   3. D_i = sum_h delta_{h,i} token by token, sum (D_i - K), sum (D_i - K)^2 about the D of the position's first
//      token;  -- barrier --  thread 0 writes the position's outputs.
// Token arithmetic is fp32 throughout: calls whose flat rows need fp64 tokens (needs_flat_pass: wide intervals on
// nearly uniform rows) are not taken by this kernel, see ensemble_fused_fits.
constexpr int kFusedHeads = 3;
constexpr int kFusedThreads = 512;
constexpr int kFusedWaves = kFusedThreads / 64;

template <typename T, int NVEC, int H, bool ARGMAX>
__global__ __launch_bounds__(kFusedThreads) __attribute__((amdgpu_waves_per_eu(4)))
void ensemble_fused_kernel(const RowArgs A, const int64_t head_stride)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec, EPT = NVEC * EPV, NW = kFusedWaves;
    constexpr int RH = H < 3 ? H : 2;                              // heads whose exponentials stay in registers
    constexpr bool LH = H == 3;                                    // the third head's go through LDS
    extern __shared__ u32x4 sm_e2[];                               // LH: [EPT / 4][kFusedThreads]
    __shared__ float sm_ref[H][NW][2];                             // per head and wave: largest logit, reference n_w
    __shared__ double sm_S[H][NW];                                 // S_w in units of 2^-n_w
    __shared__ double sm_cap[H][NW][2];                            // sum gl, sum gw of a wave, in row units of e
    __shared__ double sm_red[2][NW];
    __shared__ double sm_Sh[H], sm_alh[H], sm_auh[H];              // per head, for the loops over a run-time h
    __shared__ float sm_nh[H];
    __shared__ float sm_pm[NW];
    __shared__ int sm_pi[NW];

    // (the wave's index lives in a scalar register and the lane's index is asked for again for every position: no
    // vector register is held for them)
    const int wave_s = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int V = A.V;
    const int nvec = (V + EPV - 1) / EPV;
    const bool partial = V < NVEC * kFusedThreads * EPV;           // the row does not fill the tile

    // Wave priority by progress, as in the streaming kernel: the two workgroups of a compute unit are served oldest
    // first; the one behind gets the higher priority, so that they end together.  (32-bit row arithmetic: scalar.)
    const uint32_t n_rows = (uint32_t)A.N, g_step = gridDim.x;
    const uint32_t my_cnt = blockIdx.x < n_rows ? (n_rows - blockIdx.x + g_step - 1u) / g_step : 0u;
    uint32_t done = 0;
    for (int64_t row = blockIdx.x; row < A.N; row += gridDim.x, ++done) {
        if (my_cnt > 1u) {
            if (done < ((my_cnt + 3u) >> 2)) __builtin_amdgcn_s_setprio(3);
            else if (done < ((my_cnt + 1u) >> 1)) __builtin_amdgcn_s_setprio(2);
            else if (done < ((3u * my_cnt + 3u) >> 2)) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        // (the lane's offsets are formed anew for every position: hoisted out of the loop they would occupy registers
        // for the whole kernel)
        // (likewise the radius constants: what is derived from them is cheap, and uniform)
        uint32_t ones = ~0u;
        double ra = A.a, rb = A.b;
        asm volatile("" : "+s"(ones), "+s"(ra), "+s"(rb));
        const int lane = (int)__builtin_amdgcn_mbcnt_hi(ones, __builtin_amdgcn_mbcnt_lo(ones, 0u));
        const int wave = wave_s, t = wave_s * 64 + lane;
        // one head's row of this position goes in flight (a scalar base address and a 32-bit lane offset)
        auto request = [&](u32x4 (&buf)[NVEC], int h) {
            const uint64_t b = (uint64_t)(static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride);
            const uint32_t blo = __builtin_amdgcn_readfirstlane((uint32_t)b);
            const uint32_t bhi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
            const gbytes base = (gbytes)(((uint64_t)bhi << 32) | blo);
            if (partial) {
#pragma unroll
                for (int j = 0; j < NVEC; ++j) {
                    const uint32_t off = (uint32_t)min(j * kFusedThreads + t, nvec - 1) * 16u;
                    buf[j] = __builtin_nontemporal_load((gvec)(base + off));
                }
            } else {
                const uint32_t off = (uint32_t)t * 16u;
#pragma unroll
                for (int j = 0; j < NVEC; ++j)
                    buf[j] = __builtin_nontemporal_load((gvec)(base + (uint64_t)j * (kFusedThreads * 16u) + off));
            }
        };
        // ---- 1: a head's row as it arrives: per-wave maximum, exponentials about the wave's integer reference, S_w
        auto stats = [&](u32x4 (&buf)[NVEC], float (&e)[EPT], int h, float& emax_w) -> float {
            if (partial) {
#pragma unroll
                for (int j = 0; j < NVEC; ++j) E::mask_tail(buf[j], (j * kFusedThreads + t) * EPV, V);
            }
#pragma unroll
            for (int j = 0; j < NVEC; ++j) E::unpack(buf[j], &e[j * EPV]);
            float ml = e[0];
#pragma unroll
            for (int i = 1; i < EPT; ++i) ml = fmaxf(ml, e[i]);
            const float mw = wave_max(ml);
            const float nw = ref_of(mw);
            const float nref = nw == -INFINITY ? 0.f : nw;
            double sacc = 0.0;                                     // (one accumulator: registers are scarcer here than issue slots)
#pragma unroll
            for (int j = 0; j < NVEC; ++j) {
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    e[j * EPV + k] = exp2_ref(e[j * EPV + k], nref);
                    sacc += (double)e[j * EPV + k];
                }
                __builtin_amdgcn_sched_barrier(0);                 // keep the working set to one vector at a time
            }
            const double Sw = wave_sum(sacc);
            if (lane == 0) { sm_ref[h][wave][0] = mw; sm_ref[h][wave][1] = nw; sm_S[h][wave] = Sw; }
            emax_w = uniform_f(exp2_ref(mw, nref));                // the wave's largest e_i, in its own units
            return uniform_f(nw);
        };
        float e[RH][EPT];
        float nwv[H], emw[H];
        if constexpr (LH) {
            // the third head first: its exponentials leave for LDS, and the second head's row is requested into
            // the registers that this frees
            u32x4 b0[NVEC];
            {
                u32x4 b2[NVEC];
                request(b2, 2);
                request(b0, 0);
                float e2[EPT];
                nwv[2] = stats(b2, e2, 2, emw[2]);
#pragma unroll
                for (int q = 0; q < EPT / 4; ++q) {
                    u32x4 w;
                    w.x = __float_as_uint(e2[q * 4]); w.y = __float_as_uint(e2[q * 4 + 1]);
                    w.z = __float_as_uint(e2[q * 4 + 2]); w.w = __float_as_uint(e2[q * 4 + 3]);
                    sm_e2[q * kFusedThreads + t] = w;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            nwv[0] = stats(b0, e[0], 0, emw[0]);
            __builtin_amdgcn_sched_barrier(0);
            u32x4 b1[NVEC];
            request(b1, 1);
            __builtin_amdgcn_sched_barrier(0);
            nwv[1] = stats(b1, e[1], 1, emw[1]);
        } else {
            u32x4 buf[RH][NVEC];
#pragma unroll
            for (int h = 0; h < RH; ++h) request(buf[h], h);
#pragma unroll
            for (int h = 0; h < RH; ++h) nwv[h] = stats(buf[h], e[h], h, emw[h]);
        }
        // element i of head h as this lane holds it
        auto e_of = [&](int h, int i, const u32x4& from_lds) -> float {
            if (h < RH) return e[h][i];
            const int c = i & 3;
            return __uint_as_float(c == 0 ? from_lds.x : c == 1 ? from_lds.y : c == 2 ? from_lds.z : from_lds.w);
        };
        __syncthreads();
        // ---- 2: every head's S and reference; which heads can have an active cap ---------------------------------
        double S[H];                                               // in units of 2^-n
        float n[H];
        bool all_capless = true, any_split = false;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            float mc = sm_ref[h][0][0], nn = sm_ref[h][0][1];
#pragma unroll
            for (int w = 1; w < NW; ++w) { mc = fmaxf(mc, sm_ref[h][w][0]); nn = fmaxf(nn, sm_ref[h][w][1]); }
            double s = 0.0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float rn = sm_ref[h][w][1];
                if (rn != -INFINITY) s += sm_S[h][w] * pow2_of(rn - nn);
            }
            S[h] = uniform_d(s); n[h] = uniform_f(nn);
            const double emax = (double)exp2_ref(uniform_f(mc), n[h]);
            all_capless = all_capless && (!A.normalize || emax <= A.capless_xmax * S[h]);
            any_split = any_split || emax > 0.5 * S[h];
            __builtin_amdgcn_sched_barrier(0);                     // one head at a time: the LDS reads of all heads at once
                                                                   // would need registers that hold the rows
        }
        // this wave's units: its e_i are 2^(n - n_w) times the row's, and so is the partition sum it divides by
        double Sw_units[H];
#pragma unroll
        for (int h = 0; h < H; ++h)
            Sw_units[h] = nwv[h] != -INFINITY ? uniform_d(S[h] * pow2_any(n[h] - nwv[h])) : 1.0;
        double al[H], au[H];
#pragma unroll
        for (int h = 0; h < H; ++h) { al[h] = 1.0; au[h] = 1.0; }
        if (!all_capless) {                                        // uniform over the workgroup
            // sum p^l and sum of the widths of every head -> that head's caps
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const FuseRow fr = uniform_fr(fuse_row(Sw_units[h], ra, rb));
                double g0 = 0.0, g1 = 0.0;
#pragma unroll
                for (int q = 0; q < EPT / 4; ++q) {
                    u32x4 w = {0u, 0u, 0u, 0u};
                    if (h >= RH) w = sm_e2[q * kFusedThreads + t];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        float gl, gw;
                        fuse_token(e_of(h, q * 4 + c, w), fr, gl, gw);
                        g0 += (double)gl; g1 += (double)gw;        // (a slot past the row's end holds e = 0: gl = gw = 0)
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // back to row units of e: a power of two
                const double fw = nwv[h] != -INFINITY ? pow2_of(nwv[h] - n[h]) : 0.0;
                g0 = wave_sum(g0) * fw; g1 = wave_sum(g1) * fw;
                if (lane == 0) { sm_cap[h][wave][0] = g0; sm_cap[h][wave][1] = g1; }
            }
            __syncthreads();
#pragma unroll
            for (int h = 0; h < H; ++h) {
                double sgl = 0.0, sgw = 0.0;
#pragma unroll
                for (int w = 0; w < NW; ++w) { sgl += sm_cap[h][w][0]; sgw += sm_cap[h][w][1]; }
                const double Sl = fmin(1.0, rb / S[h] * sgl), Su = fmax(1.0, rb / S[h] * sgl + (ra - rb) / S[h] * sgw);
                if (A.normalize) { al[h] = uniform_d(fmin(1.0, A.cap_lo / Sl)); au[h] = uniform_d(fmax(1.0, A.cap_hi / Su)); }
            }
        }
        if (t == 0) {
#pragma unroll
            for (int h = 0; h < H; ++h) { sm_Sh[h] = S[h]; sm_nh[h] = n[h]; sm_alh[h] = al[h]; sm_auh[h] = au[h]; }
        }
        // The sums over the tokens are taken about the D of the position's first token (every lane forms the same
        // number, from the logits in memory and the row's constants).
        double KD = 0.0;
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const T* crow = static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride;
            const float e0 = exp2_ref(load_logit(crow, 0), n[h]);
            float gl, gw;
            fuse_token(e0, fuse_row(S[h], ra, rb), gl, gw);
            KD = fma(au[h] * (ra - rb) / S[h], (double)gw, fma((au[h] - al[h]) * rb / S[h], (double)gl, KD));
        }
        KD = uniform_d(KD);
        double s1 = 0.0, s2 = 0.0;
        float best = -INFINITY;
        int best_i = INT_MAX;
        {
            // ---- 3: D_i in this wave's units of every head ---------------------------------------------------------
            FuseRow fr[H];
            double cw[H], cl[H];
            float invS[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                fr[h] = uniform_fr(fuse_row(Sw_units[h], ra, rb));
                cw[h] = uniform_d(au[h] * (ra - rb) / Sw_units[h]);
                cl[h] = uniform_d((au[h] - al[h]) * rb / Sw_units[h]);
                invS[h] = uniform_f((float)(1.0 / Sw_units[h]));
            }
            // Specialised on what is uniform over the position or the wave: NOLOW = no head has an active cap (delta = w:
            // p^l is not needed), SPLIT = some probability above 1/2 (1 - x needs the two-float 1/S, see fuse_parts),
            // POLY = every token this wave holds, in every head, is small enough for the width polynomial that the host
            // has fitted for the call's radius (gw = e (1 + x P(x)), see RowArgs::wpoly): five FMAs instead of the
            // rational form with its reciprocal.
            float pd[H][4];
            bool poly = all_capless && A.wpoly_x >= 0.f;
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float is = -fr[h].nih, is2 = is * is;
                pd[h][0] = uniform_f(A.wpoly[0] * is); pd[h][1] = uniform_f(A.wpoly[1] * is2);
                pd[h][2] = uniform_f(A.wpoly[2] * (is2 * is)); pd[h][3] = uniform_f(A.wpoly[3] * (is2 * is2));
                poly = poly && (double)emw[h] <= (double)A.wpoly_x * Sw_units[h];
            }
            auto sweep = [&](auto nolow_c, auto split_c, auto poly_c) {
                constexpr bool NOLOW = decltype(nolow_c)::value, SPLIT = decltype(split_c)::value;
                constexpr bool POLY = decltype(poly_c)::value;
#pragma unroll
                for (int q = 0; q < EPT / 4; ++q) {
                    const int j = q * 4 / EPV;
                    if (j * kFusedThreads * EPV >= V) continue;      // uniform: the chunk holds no token
                    u32x4 w = {0u, 0u, 0u, 0u};
                    if constexpr (LH) w = sm_e2[q * kFusedThreads + t];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int i = q * 4 + c;
                        double D = 0.0;
                        float pm = 0.f;
#pragma unroll
                        for (int h = 0; h < H; ++h) {
                            const float eh = e_of(h, i, w);
                            if constexpr (POLY) {
                                const float G = fmaf(fmaf(fmaf(fmaf(pd[h][3], eh, pd[h][2]), eh, pd[h][1]), eh, pd[h][0]), eh, 1.0f);
                                D = fma(cw[h], (double)(eh * G), D);
                            } else {
                                float g, du, om;
                                fuse_parts<SPLIT>(eh, fr[h], g, du, om);
                                D = fma(cw[h], (double)(g * om), D);
                                if constexpr (!NOLOW) D = fma(cl[h], (double)(g * du), D);
                            }
                            if (ARGMAX) pm = fmaf(eh, invS[h], pm);
                        }
                        // A slot past the row's end holds e = 0 in every head: D = 0 exactly, so it adds -KD and KD^2
                        // to the two sums, which thread 0 takes out again (the number of such slots is known); its mean
                        // probability 0 never wins the arg-max (strict comparison, and the lane's real tokens come first).
                        const double d = D - KD;
                        s1 += d;
                        s2 = fma(d, d, s2);
                        if (ARGMAX && pm > best) { best = pm; best_i = (j * kFusedThreads + t) * EPV + (i - j * EPV); }
                        if (c & 1) __builtin_amdgcn_sched_barrier(0);  // two tokens at a time: bounded working set
                    }
                }
            };
            using yes = std::integral_constant<bool, true>;
            using no = std::integral_constant<bool, false>;
            if (poly) sweep(yes{}, no{}, yes{});                    // (uniform over the wave)
            else if (all_capless) { if (any_split) sweep(yes{}, yes{}, no{}); else sweep(yes{}, no{}, no{}); }
            else { if (any_split) sweep(no{}, yes{}, no{}); else sweep(no{}, no{}, no{}); }
        }
        s1 = wave_sum(s1);
        s2 = wave_sum(s2);
        if (lane == 0) { sm_red[0][wave] = s1; sm_red[1][wave] = s2; }
        if (ARGMAX) {
            // each lane walked its tokens in ascending order, so it holds its lowest index of its maximum
            const float wm = wave_max(best);
            const int wi = wave_min_i(best == wm ? best_i : INT_MAX);
            if (lane == 0) { sm_pm[wave] = wm; sm_pi[wave] = wi; }
        }
        __syncthreads();
        if (t == 0) {
            int Vr = V;
            asm volatile("" : "+s"(Vr));                           // (so that its conversion stays in this block)
            const double Hd = (double)H, Vd = (double)Vr;
            double t1 = 0.0, t2 = 0.0;
            for (int w = 0; w < NW; ++w) { t1 += sm_red[0][w]; t2 += sm_red[1][w]; }
            {
                // the slots of the tile past the row's end (chunks that hold no token at all were skipped)
                const int chunks = (Vr + kFusedThreads * EPV - 1) / (kFusedThreads * EPV);
                const double pad = (double)(chunks * kFusedThreads * EPV - Vr);
                t1 += pad * KD;
                t2 -= pad * KD * KD;
            }
            const double omega = (t1 + Vd * KD) / Hd;
            const double var = fmax(0.0, t2 - t1 * t1 / Vd) / (Hd * Hd * Vd);
            const double sigma = sqrt(var), score = omega * sigma;
            if (A.omega) A.omega[row] = (float)omega;
            if (A.sigma) A.sigma[row] = (float)sigma;
            if (A.score) A.score[row] = (float)score;
            if (A.flags) A.flags[row] = (uint8_t)(score > A.tau);
            if (A.p_lo || A.p_mid || A.p_hi) {
                int xid;
                if (A.ids) {
                    xid = A.ids[row];
                    xid = xid < 0 ? 0 : (xid >= V ? V - 1 : xid);
                } else {
                    float rm = sm_pm[0];
                    for (int w = 1; w < NW; ++w) rm = fmaxf(rm, sm_pm[w]);
                    xid = INT_MAX;
                    for (int w = 0; w < NW; ++w) if (sm_pm[w] == rm && sm_pi[w] < xid) xid = sm_pi[w];
                    if (xid == INT_MAX) xid = 0;
                }
                double lo = 0.0, mid = 0.0, hi = 0.0;
#pragma nounroll
                for (int h = 0; h < H; ++h) {
                    const T* crow = static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride;
                    const double Sh = sm_Sh[h];
                    const double ex = (double)exp2_ref(load_logit(crow, xid), sm_nh[h]);
                    const double x = ex / Sh, omx = fmax(0.0, Sh - ex) / Sh;
                    mid += x;
                    lo += sm_alh[h] * rb * x / (rb + (1.0 - rb) * omx);
                    hi += sm_auh[h] * ra * x / (1.0 + (ra - 1.0) * x);
                }
                if (A.p_lo) A.p_lo[row] = (float)(lo / Hd);
                if (A.p_mid) A.p_mid[row] = (float)(mid / Hd);
                if (A.p_hi) A.p_hi[row] = (float)(hi / Hd);
            }
        }
        // (the next position's first barrier separates this read of sm_red / sm_pm from their next writes)
    }
}

// Voting: flags[row] = strict majority of head_flags[h][row].
__global__ __launch_bounds__(256) void vote_kernel(const uint8_t* __restrict__ head_flags, int H, int64_t N,
                                                   uint8_t* __restrict__ flags)
{
    const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (row >= N) return;
    int votes = 0;
    for (int h = 0; h < H; ++h) votes += head_flags[(int64_t)h * N + row] != 0;
    flags[row] = (uint8_t)(2 * votes > H);
}

}  // namespace

int max_heads() { return kMaxHeads; }

hipError_t launch_ensemble(int dtype, const RowArgs& args, int heads, int64_t head_stride, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)args.N), block(256);
    if (wide_radius(args)) {
        if (dtype == 0) hipLaunchKernelGGL((ensemble_kernel<float, true>), grid, block, 0, stream, args, heads, head_stride);
        else hipLaunchKernelGGL((ensemble_kernel<bf16_t, true>), grid, block, 0, stream, args, heads, head_stride);
    } else {
        if (dtype == 0) hipLaunchKernelGGL((ensemble_kernel<float, false>), grid, block, 0, stream, args, heads, head_stride);
        else hipLaunchKernelGGL((ensemble_kernel<bf16_t, false>), grid, block, 0, stream, args, heads, head_stride);
    }
    return hipGetLastError();
}

bool ensemble_fused_fits(int dtype, const RowArgs& args, int heads)
{
    if (args.radius || wide_radius(args) || needs_flat_pass(args) || heads < 1 || heads > kFusedHeads || args.V <= 64) return false;
    const int epv = dtype == 0 ? 4 : 8;
    const int nvec = (args.V + epv - 1) / epv;
    const int per_lane = (nvec + kFusedThreads - 1) / kFusedThreads * epv;   // elements of one head's row per lane
    return per_lane <= 32;
}

namespace {
template <typename T, int NVEC, int H>
hipError_t launch_ensemble_fused_heads(const RowArgs& a, int64_t head_stride, hipStream_t stream)
{
    const int64_t resident = 2 * (int64_t)compute_units();
    const dim3 grid((unsigned)(a.N < resident ? a.N : resident)), block(kFusedThreads);
    const bool argmax = a.ids == nullptr && (a.p_lo || a.p_mid || a.p_hi);
    // the third head's exponentials: 4 bytes x elements per lane x lanes (64 KiB for the largest tile), above the
    // default limit on dynamic LDS together with the static arrays: raised once per device and instance
    constexpr unsigned lds = H == 3 ? NVEC * Elt<T>::kPerVec * kFusedThreads * 4u : 0u;
    if (lds) {
        static std::mutex guard;
        static bool raised[2][64] = {};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
        std::lock_guard<std::mutex> lock(guard);
        if (!raised[argmax ? 1 : 0][dev]) {
            const hipError_t e = argmax
                ? hipFuncSetAttribute(reinterpret_cast<const void*>(&ensemble_fused_kernel<T, NVEC, H, true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                : hipFuncSetAttribute(reinterpret_cast<const void*>(&ensemble_fused_kernel<T, NVEC, H, false>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            raised[argmax ? 1 : 0][dev] = true;
        }
    }
    if (argmax) hipLaunchKernelGGL((ensemble_fused_kernel<T, NVEC, H, true>), grid, block, lds, stream, a, head_stride);
    else hipLaunchKernelGGL((ensemble_fused_kernel<T, NVEC, H, false>), grid, block, lds, stream, a, head_stride);
    return hipGetLastError();
}
template <typename T, int NVEC>
hipError_t launch_ensemble_fused_cfg(const RowArgs& a, int heads, int64_t head_stride, hipStream_t stream)
{
    static_assert(kFusedHeads == 3, "one instance per number of heads");
    if (heads == 1) return launch_ensemble_fused_heads<T, NVEC, 1>(a, head_stride, stream);
    if (heads == 2) return launch_ensemble_fused_heads<T, NVEC, 2>(a, head_stride, stream);
    return launch_ensemble_fused_heads<T, NVEC, 3>(a, head_stride, stream);
}
}  // namespace

hipError_t launch_ensemble_fused(int dtype, const RowArgs& args, int heads, int64_t head_stride, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    if (!ensemble_fused_fits(dtype, args, heads)) return hipErrorInvalidValue;
    const int epv = dtype == 0 ? 4 : 8;
    const int nvec = (args.V + epv - 1) / epv;
    const int per_lane = (nvec + kFusedThreads - 1) / kFusedThreads;
    if (dtype == 0) {
        if (per_lane <= 2) return launch_ensemble_fused_cfg<float, 2>(args, heads, head_stride, stream);
        if (per_lane <= 4) return launch_ensemble_fused_cfg<float, 4>(args, heads, head_stride, stream);
        return launch_ensemble_fused_cfg<float, 8>(args, heads, head_stride, stream);
    }
    if (per_lane <= 2) return launch_ensemble_fused_cfg<bf16_t, 2>(args, heads, head_stride, stream);
    return launch_ensemble_fused_cfg<bf16_t, 4>(args, heads, head_stride, stream);
}

hipError_t launch_vote(const uint8_t* head_flags, int heads, int64_t N, uint8_t* flags, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(vote_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, stream, head_flags, heads, N, flags);
    return hipGetLastError();
}

}  // namespace ciar
