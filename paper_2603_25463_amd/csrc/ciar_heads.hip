// gfx950 kernels for several Interval Heads (Sec. 4, ablation on the Inter-Head): the Ensemble sweep that
// averages the heads' widths token by token, and the Voting majority.
#include "ciar_device.h"

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
    for (int h = 0; h < H; ++h) {
        const T* crow = static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride;
        const T* rrow = static_cast<const T*>(rad ? A.radius : A.draft) + (int64_t)h * head_stride + row * A.stride;
        const float c0 = load_logit(crow, 0), r0 = load_logit(rrow, 0);
        if (precise) head_token_tiny(h, c0, r0, KD, KC);
        else head_token(h, c0, r0, sm_fr[h], KD, KC);
    }
    double s1 = 0.0, s2 = 0.0;                                     // sum (D_i - KD), sum (D_i - KD)^2
    double c1 = 0.0, c2 = 0.0, cbig = 0.0;                         // WIDE: sum (C_i - KC), its square, max C_i
    float best = -INFINITY;
    int best_i = INT_MAX;
    if (precise) {
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
    }
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

hipError_t launch_vote(const uint8_t* head_flags, int heads, int64_t N, uint8_t* flags, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(vote_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, stream, head_flags, heads, N, flags);
    return hipGetLastError();
}

}  // namespace ciar
