// gfx950 kernels for the forward value of the Inter-DRO loss (Sec. 3.2.3: anchor, DRO and alignment
// equations): per-row terms, batch softmax weights and the batch reduction.
#include "ciar_device.h"

#include <cfloat>
#include <mutex>

namespace ciar {
namespace {

// ---- Inter-DRO loss, forward (Sec. 3.2.3: anchor, DRO and alignment equations) -----------------------------

// The distributions over c + r and c - r are taken about a reference pair (cs, rs) from the differences c - cs and
// r - rs: each is exact for tokens near the reference and rounded relative to itself elsewhere, so c + r is never
// rounded to fp32.  That rounding, 6e-8 |c + r|, would be a relative error of the same size in the token's
// probability, and for logits of magnitude ~30 it shows as ~1e-6 absolute in a cross-entropy and in an L1 distance.
//
// The exponentials of c + r and c - r are formed as products, e^(c - cs) e^(r - rs) and e^(c - cs) e^-(r - rs), not from
// the sums of the exponents: where the radius is the same for every token of a row (scalar mode, or a row clamped at
// r_max) r - rs is one number, and adding it to exponents of one binade rounds them all the same way -- by up to half
// an ulp of that binade, another amount in the next one.  That tilts the distribution between the binades by up to
// ~3e-7 of the mass they hold, upwards for c + r and downwards for c - r, and showed as 1.7e-7 absolute in an L1
// distance of 6e-3 (a seeded random case).  As products the three distributions of such a row agree to the rounding
// of single tokens.  |r - rs| <= r_max <= 16: the factors stay within 2^+-24.
struct RadiusFactors { float up, lo; };
__device__ __forceinline__ RadiusFactors radius_factors(float r, float rs)
{
    const float d = r - rs, x = fmaf(d, kLog2eLo, d * kLog2eHi);
    return {__builtin_amdgcn_exp2f(x), __builtin_amdgcn_exp2f(-x)};
}

// r = min(kappa Softplus(raw), rmax) to the rounding of r itself (radius_r keeps small radii accurate relative to
// themselves, which the interval widths need; here the radius only shifts logits, and the shorter form saves
// instructions): Softplus(raw) = max(raw, 0) + ln(1 + t), t = e^-|raw|.  The sum u = 1 + t rounds t to half an ulp of u,
// 6e-8 absolute -- kappa times that in the radius, and a radius that is off by d moves the probability p of its token
// under c + r and c - r by p (1 - p) d in opposite directions: with kappa = 3.9 and two tokens of p ~ 1/2 an L1
// distance of 2.5e-3 came out 1.9e-7 off (a seeded random case).  What the sum lost, t - (u - 1), is exact in fp32
// and is given back to first order, ln(1 + t) = ln u + (t - (u - 1)) / u + ...; for 1 / u a line over [1, 2] is enough
// (within 9 %: the term is at most 6e-8).
__device__ __forceinline__ float radius_abs(float raw, float kappa, float rmax)
{
    const float t = __builtin_amdgcn_exp2f(-fabsf(raw) * 1.44269504f);
    const float u = 1.0f + t;
    const float lost = t - (u - 1.0f);
    const float ln1p = fmaf(__builtin_amdgcn_logf(u), 0.693147181f, lost * fmaf(-0.5f, u, 1.4571f));
    return fminf(kappa * (ln1p + fmaxf(raw, 0.f)), rmax);
}

// e^(x - m) for a row of plain logits.
__device__ __forceinline__ float exp_rel(float x, float m)
{
    const float d = x - m;
    return __builtin_amdgcn_exp2f(fmaf(d, kLog2eLo, d * kLog2eHi));
}

// Stand-in for a centre logit of -inf inside dro_row_compute: -2^100, a bf16 and an fp32 number whose multiples by
// log2(e) and differences from any logit stay finite.
constexpr float kRuledOut = -1267650600228229401496703205376.0f;
constexpr uint32_t kRuledOutBits = 0xf1800000u;                    // (its upper half is the bf16 number)

// Per-row terms of the loss.  One 1024-lane workgroup per row holds the centre, raw-radius and cloud rows as
// loaded (12 registers per vector) and makes three passes over them: the maxima of the centre and the cloud logits
// and a reference radius, the four partition sums together with the p_cloud-weighted sums of the exponents for the
// cross-entropies, and the three L1 distances, which need all four normalisers.  With e = exp(o - reference):
//   CE(p_cloud, softmax(o)) = (reference + ln S_o) - (sum_i et_i o_i) / Z,
//   KL(p_cloud || p_mid)    = ln S_mid - ln Z + (sum_i et_i ((t_i - max t) - (c_i - max c))) / Z.
// terms[k * N + row], k = 0..6: L1(mid), L1(up), L1(lo), CE(mid), CE(up), CE(lo), KL.
// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS operations and joins the barrier.
// __syncthreads() would also wait for every outstanding global load (its fence covers all memory), and with it for
// the next row that dro_row_stream_kernel has in flight while it works on the current one.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One row's totals (see dro_finish_row) from the three rows as loaded (lane t holds 16-byte vectors j * 1024 + t;
// vectors past the end of the row hold copies of its last vector and are masked here), left in fin[kDroTotals] (LDS)
// by lane 0.  Called by every lane of a 1024-lane workgroup; sm_d: 7 doubles per wave of LDS scratch.  Ends with every
// lane past the last read of sm_d except wave 0's.
// The radius parameters as the row arithmetic takes them: floats, formed by the host, so that they arrive in scalar
// registers with the kernel arguments.  (Converted from RowArgs' doubles inside a kernel they are loop invariants that
// the optimiser holds in vector registers, or spills, through the whole row loop.)
struct DroRadius { float kappa, rmax, scalar; };                   // scalar = min(kappa, rmax), the radius without a tensor

template <typename T, int NVEC>
__device__ __forceinline__ void dro_row_compute(const RowArgs& A, const DroRadius R, double* fin,
                                                u32x4 (&cw)[NVEC], u32x4 (&tw)[NVEC], u32x4 (&rw)[NVEC], double* sm_d,
                                                const int tid)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec, THREADS = 1024, NW = 16;
    const int lane = tid & 63, wave = tid >> 6;
    const int V = A.V;
    const bool rad = A.radius != nullptr;                          // uniform
    auto uniform = [](float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); };
    const float kap = R.kappa, rmax = R.rmax, r0 = R.scalar;
    if (V < NVEC * THREADS * EPV) {                                // uniform: the row does not fill the tile
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            const int base = (j * THREADS + tid) * EPV;
            E::mask_tail(cw[j], base, V);
            E::mask_tail(tw[j], base, V);
            if (rad) E::zero_tail(rw[j], base, V);
        }
    }
    // The radii are formed once (Softplus costs about as much as the rest of a pass) and kept as floats where
    // the registers allow: up to 32 tokens per lane.  Beyond that they are recomputed in every pass.
    constexpr bool CACHE_R = NVEC * EPV <= 32;
    float rc[CACHE_R ? NVEC * EPV : 1];
    if constexpr (CACHE_R) {
        if (rad) {                                                 // (one branch for the row, not one per token)
#pragma unroll
            for (int j = 0; j < NVEC; ++j) {
                float rv[EPV];
                E::unpack(rw[j], rv);
#pragma unroll
                for (int k = 0; k < EPV; ++k) rc[j * EPV + k] = radius_abs(rv[k], kap, rmax);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NVEC * EPV; ++i) rc[i] = r0;
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
            if (rad) { E::unpack(rw[j], rv); r = radius_abs(rv[k], kap, rmax); }
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
    // pass 1: the maxima of c and of the cloud logits, and a reference radius r* for the sums of c + r and c - r: the
    // radius of a token at (or within 2^-11 of) the maximum of c.  Any reference gives the same cross-entropy
    //   CE = ln S - (sum_i et_i d_i) / Z,   S and the d_i taken about the same one,
    // but its two terms cancel down from the size of the dominant token's exponent, and the weighted sum is rounded
    // per lane in fp32: with r* the radius of that very token its exponent is ~0 in all three distributions (where
    // the cloud puts its weight elsewhere, the cross-entropy is large and the rounding small beside it).  The
    // exponents are then (c - max c) +- (r - r*) <= r_max <= 16: nothing overflows, and the token at the maximum
    // keeps every partition sum above ~1.
    // r* comes out of the same maximum: the key of a token is its centre logit with the low 12 mantissa bits replaced
    // by the radius in 1/128ths (the low bits of r + 2^16), so the largest key carries the radius of a largest logit.
    auto key_of = [](float c, float r) {
        return __uint_as_float((__float_as_uint(c) & 0xFFFFF000u) | (__float_as_uint(r + 65536.0f) & 0x00000FFFu));
    };
    // (the keys are ordered as floats, none is a NaN: plain v_max_f32, without the quieting of its operands that
    // fmaxf adds for values the compiler knows nothing about)
    auto key_max = [](float a, float b, float c) {
        float m;
        asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m) : "v"(a), "v"(b), "v"(c));
        return m;
    };
    float mc = -INFINITY, mt = -INFINITY, key = -FLT_MAX;
    float c_least = INFINITY;                                      // (this lane's smallest centre logit: see pass 2)
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
#pragma unroll
        for (int k = 0; k < EPV; k += 2) {
            float c, r, t, c2, r2, t2;
            element(j, k, c, r, t);
            element(j, k + 1, c2, r2, t2);
            mc = fmaxf(fmaxf(mc, c), c2); mt = fmaxf(fmaxf(mt, t), t2);
            c_least = fminf(fminf(c_least, c), c2);
            key = key_max(key, key_of(c, r), key_of(c2, r2));
        }
    }
    // Does any lane of this wave hold a centre logit of -inf (a token the device rules out, or the masked tail)?  Its
    // key would be a NaN, and in pass 2 its exponent times a cloud weight of 0 another.  Such a wave (only such a wave)
    // puts kRuledOut, a finite number far below any logit, in the place of -inf in the row as it holds it and forms its
    // key again; pass 2 then sees finite numbers only.  (A logit of exactly kRuledOut counts as ruled out.)
    const bool wave_c_finite = __builtin_amdgcn_ballot_w64(c_least == -INFINITY) == 0;
    if (!wave_c_finite) {
        key = -FLT_MAX;
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            uint32_t* w = reinterpret_cast<uint32_t*>(&cw[j]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if constexpr (EPV == 4) {
                    if (w[q] == 0xff800000u) w[q] = kRuledOutBits;
                } else {                                           // two bf16 numbers to a word
                    if ((w[q] & 0x0000ffffu) == 0x0000ff80u) w[q] = (w[q] & 0xffff0000u) | (kRuledOutBits >> 16);
                    if ((w[q] & 0xffff0000u) == 0xff800000u) w[q] = (w[q] & 0x0000ffffu) | kRuledOutBits;
                }
            }
#pragma unroll
            for (int k = 0; k < EPV; k += 2) {
                float c, r, t, c2, r2, t2;
                element(j, k, c, r, t);
                element(j, k + 1, c2, r2, t2);
                key = key_max(key, key_of(c, r), key_of(c2, r2));
            }
        }
    }
    // LDS for the reductions over the workgroup (see pass 2 for the scheme: quad sums by DPP, then transposed through
    // LDS so that one short reduction serves all quantities at once)
    __shared__ __attribute__((aligned(16))) double sm_w[NW][8][16];   // per wave: [quantity][quad]
    __shared__ __attribute__((aligned(16))) double sm_x[8][16];       // [quantity][wave]
    float rref;
    {
        // the four maxima over the workgroup: quads by DPP, the 16 quad maxima of each quantity through LDS into one
        // DPP row each (lanes 16 q ... 16 q + 15 take quantity q), one row reduction for all four; the same again
        // over the sixteen waves.  (Four wave-wide DPP maxima, twice, cost ~240 instructions.)
        float m4[4] = {mc, mt, key, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            m4[i] = dpp_max<0xB1, 0xf>(m4[i]);
            m4[i] = dpp_max<0x4E, 0xf>(m4[i]);
        }
        float* fw = reinterpret_cast<float*>(&sm_w[wave][0][0]);   // [4][16] floats of this wave
        __shared__ float sm_m[4 * 16];                             // [quantity][wave], this step's own (no barrier behind it)
        float* fx = sm_m;
        if ((lane & 3) == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) fw[i * 16 + (lane >> 2)] = m4[i];
        }
        auto row_max = [](float v) {                               // lane 15 of each DPP row: the row's maximum
            v = dpp_max<kRowShr1, 0xf>(v);
            v = dpp_max<kRowShr2, 0xf>(v);
            v = dpp_max<kRowShr4, 0xf>(v);
            v = dpp_max<kRowShr8, 0xf>(v);
            return v;
        };
        float v = row_max(fw[lane]);                               // (= fw[(lane >> 4) * 16 + (lane & 15)])
        if ((lane & 15) == 15) fx[(lane >> 4) * 16 + wave] = v;
        lds_barrier();
        v = row_max(fx[lane]);
        mc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
        mt = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
        rref = (float)(__builtin_amdgcn_readlane(__float_as_int(v), 47) & 0xFFF) * (1.0f / 128.0f);
        // (sm_m is written again in the next row's pass 1, with the barriers of passes 2 and 3 in between)
    }
    // a row without a live token: any finite reference will do (every exponential is 0)
    if (mc == -INFINITY) mc = 0.f;
    if (mt == -INFINITY) mt = 0.f;
    // the references are the same in every lane: keep them in scalar registers
    mc = uniform(mc); mt = uniform(mt); rref = uniform(rref);

    // pass 2: partition sums and the p_cloud-weighted sums of the exponents.  With d = o - reference and e = exp(d):
    //   CE(p_cloud, softmax(o)) = ln S_o - (sum_i et_i d_i) / Z;
    // for the centre and the cloud's own distribution the reference is the row maximum, d <= 0 and both terms are
    // non-negative, so nothing is lost to cancellation whatever the size of the logits (for c + r and c - r see
    // pass 1); likewise the entropy of p_cloud, H = ln Z - (sum_i et_i dt_i) / Z, and
    // KL(p_cloud || p_mid) = CE(p_cloud, p_mid) - H = ln S - ln Z + (sum_i et_i (dt_i - d_i)) / Z: the fourth weighted
    // sum is taken over the differences dt_i - d_i, so that a small KL is not the difference of two large sums.
    // With at most 16 tokens per lane the four exponentials of every token are kept for pass 3 (the rows themselves
    // are not needed again).  The partition sums run in fp64 from the first add: in a row with one dominant token the
    // lane that holds it carries nearly all of S, so a lane sum kept in fp32 would round S itself to 6e-8, and ln S
    // with it -- as much as a whole cross-entropy of such a row may be off.  The four weighted sums of exponents are
    // taken per lane in fp32 (the dominant token has exponent 0 and adds nothing to them; what a lane's rounding
    // leaves is ~1e-7 of that lane's share of a cross-entropy), and in fp64 across lanes and waves.
    constexpr bool CACHE_E = NVEC * EPV <= 16;
    constexpr int NE = CACHE_E ? NVEC * EPV : 1;
    float em[NE], eu[NE], el[NE], ec[NE];
    fresh();
    double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};     // S_mid, S_up, S_lo, Z, sum et d_mid, d_up, d_lo, d_t
    float s32[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // (x log2(e) from the two-piece constant: a single fp32 constant is off by 2e-8 of itself, the same way for every
    // token, which would tilt a distribution over logits ~10 apart by 2e-7)
    auto log2e_times = [](float d) { return fmaf(d, kLog2eLo, d * kLog2eHi); };
    // A token the cloud rules out (et = 0) weighs nothing in the weighted sums, whatever its logits are; but 0 x -inf
    // would be NaN.  So the products are formed from finite numbers: kRuledOut stands for a centre logit of -inf (see
    // pass 1) and dt has a floor of -1e30; neither changes an exponential (2^-1e30 = 0 = 2^-inf).  What that would
    // lose -- a token that the device rules out and the cloud does not makes the cross-entropies and KL infinite --
    // is looked for beforehand, by the waves that hold such a logit.
    bool ce_infinite = false;
    if (!wave_c_finite) {
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
#pragma unroll
            for (int k = 0; k < EPV; ++k) {
                float c, r, t;
                element(j, k, c, r, t);
                ce_infinite |= c == kRuledOut && __builtin_amdgcn_exp2f(log2e_times(t - mt)) > 0.f;
            }
        }
    }
    // The exponents are taken to base 2 once, x = d log2(e), and the weighted sums run over x (dro_finish_row
    // multiplies them by ln 2); x_up and x_lo are x_mid +- xa, xa = (r - r*) log2(e), so their weighted sums are those
    // of x_mid and xa added and subtracted.
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float c, r, t;
            element(j, k, c, r, t);
            // (each difference is exact for tokens near the reference and rounded relative to itself elsewhere:
            // c + r is never rounded to fp32)
            const float x0 = log2e_times(c - mc), xa = log2e_times(r - rref);
            const float xt = log2e_times(fmaxf(t - mt, -1e30f));
            // (the exponentials of c + r and c - r are products: see radius_factors)
            const float e0 = __builtin_amdgcn_exp2f(x0), et = __builtin_amdgcn_exp2f(xt);
            const float e1 = e0 * __builtin_amdgcn_exp2f(xa), e2 = e0 * __builtin_amdgcn_exp2f(-xa);
            if constexpr (CACHE_E) {
                em[j * EPV + k] = e0; eu[j * EPV + k] = e1; el[j * EPV + k] = e2; ec[j * EPV + k] = et;
                acc[0] += (double)e0; acc[1] += (double)e1; acc[2] += (double)e2; acc[3] += (double)et;
                s32[4] = fmaf(et, x0, s32[4]); s32[5] = fmaf(et, xa, s32[5]);
                s32[7] = fmaf(et, xt - x0, s32[7]);
            } else {
                acc[0] += (double)e0; acc[1] += (double)e1; acc[2] += (double)e2; acc[3] += (double)et;
                acc[4] = fma((double)et, (double)x0, acc[4]); acc[5] = fma((double)et, (double)xa, acc[5]);
                acc[7] = fma((double)et, (double)(xt - x0), acc[7]);
            }
            if (k & 1) __builtin_amdgcn_sched_barrier(0);          // two tokens at a time: bounded working set
        }
    }
    // the sums over x_up = x_mid + xa and x_lo = x_mid - xa from the sums over x_mid and xa
    {
        const float sa = s32[5];
        s32[5] = s32[4] + sa; s32[6] = s32[4] - sa;
        const double da = acc[5];
        acc[5] = acc[4] + da; acc[6] = acc[4] - da;
    }
    if (ce_infinite) {
#pragma unroll
        for (int i = 4; i < 7; ++i) { s32[i] = -INFINITY; acc[i] = -INFINITY; }
        s32[7] = INFINITY; acc[7] = INFINITY;                      // KL is infinite with the cross-entropies
    }
    if constexpr (CACHE_E) {
        // (the weighted sums of a quad in fp32 as well: one instruction per DPP step of a float, five of a double)
#pragma unroll
        for (int i = 4; i < 8; ++i) {
            float v = s32[i];
            v += __int_as_float(dpp_or<0xB1, 0xf>(0, __float_as_int(v)));
            v += __int_as_float(dpp_or<0x4E, 0xf>(0, __float_as_int(v)));
            acc[i] = (double)v;
        }
    }
    // The eight sums over the workgroup.  A DPP reduction of one double over a wave is ~36 instructions, and with 16
    // tokens per lane eight of them (and eight more across the waves) weighed more than the tokens' own arithmetic.
    // Instead: two DPP steps leave every quad's sum in its lanes; the quad leaders put them into LDS, quantity by
    // quantity; lane l then takes two of the 16 quad sums of quantity l / 8 (one 16-byte read) and three butterfly
    // steps over its group of eight lanes finish the wave's sums of all quantities at once.  Across the waves the same
    // two last steps run on the sixteen wave sums.
    const int grp = lane >> 3, part = lane & 7;
    auto group8_total = [](double a) {
        a = dpp_add<0xB1, 0xf>(a);                                 // lane ^ 1  (quad_perm 1,0,3,2)
        a = dpp_add<0x4E, 0xf>(a);                                 // lane ^ 2  (quad_perm 2,3,0,1)
        a = dpp_add<0x141, 0xf>(a);                                // the other quad of the eight (row_half_mirror)
        return a;
    };
#pragma unroll
    for (int i = 0; i < (CACHE_E ? 4 : 8); ++i) {
        acc[i] = dpp_add<0xB1, 0xf>(acc[i]);
        acc[i] = dpp_add<0x4E, 0xf>(acc[i]);
    }
    if ((lane & 3) == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) sm_w[wave][i][lane >> 2] = acc[i];
    }
    {
        // (the wave reads what its own lanes have written: LDS operations of a wave complete in order)
        const double* pr = &sm_w[wave][grp][2 * part];
        const double a = group8_total(pr[0] + pr[1]);
        if (part == 0) sm_x[grp][wave] = a;
    }
    lds_barrier();
    double tot[8];
    {
        const double* pr = &sm_x[grp][2 * part];
        const double a = group8_total(pr[0] + pr[1]);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            tot[i] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(a), 8 * i),
                                      __builtin_amdgcn_readlane(__double2loint(a), 8 * i));
    }
    // (sm_x is written again only after the next barriers: pass 3's exchange uses sm_d)

    // pass 3: L1 distances to p_cloud.  With rho = S / Z,  |e / S - et / Z| = |e - rho et| / S:  the difference is one
    // fused multiply-add on the exponentials as they are, rounded once at its own (small) size, so tokens that carry
    // most of both distributions cancel to the last bit.  rho is carried as two floats (a second multiply-add takes the
    // low part): rounded to one float it is off by up to 6e-8 of itself, which moves every term the same way -- up to
    // 6e-8 of the weight the cloud puts where the two distributions differ in one direction, and for a peaked row whose
    // distance is small that was the whole absolute tolerance (a seeded random case: distance 4.0e-4, off by 1.06e-7).
    // (A product e * (1/S) rounded on its own would leave that much per factor and per term.)
    // The division by S is left to dro_finish_row.
    float rho[3], rlo[3];
    {
        // 1 / Z: hardware reciprocal and one Newton step in fp64 (~1e-14), no fp64 division
        const double z = tot[3], r0 = (double)__builtin_amdgcn_rcpf((float)z);
        const double rz = fma(r0, fma(-z, r0, 1.0), r0);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const double rr = tot[i] * rz;
            rho[i] = (float)rr;
            rlo[i] = (float)(rr - (double)rho[i]);
        }
    }
    double l1[3] = {0.0, 0.0, 0.0};
    if constexpr (CACHE_E) {
        float a32[3] = {0.f, 0.f, 0.f};                            // (per lane in fp32: sums of non-negative terms)
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            a32[0] += fabsf(fmaf(-ec[i], rlo[0], fmaf(-ec[i], rho[0], em[i])));
            a32[1] += fabsf(fmaf(-ec[i], rlo[1], fmaf(-ec[i], rho[1], eu[i])));
            a32[2] += fabsf(fmaf(-ec[i], rlo[2], fmaf(-ec[i], rho[2], el[i])));
        }
#pragma unroll
        for (int i = 0; i < 3; ++i) l1[i] = (double)a32[i];
    } else {
        fresh();
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
#pragma unroll
            for (int k = 0; k < EPV; ++k) {
                float c, r, t;
                element(j, k, c, r, t);
                const float et = exp_rel(t, mt), e0 = exp_rel(c, mc);
                const RadiusFactors f = radius_factors(r, rref);
                l1[0] += (double)fabsf(fmaf(-et, rlo[0], fmaf(-et, rho[0], e0)));
                l1[1] += (double)fabsf(fmaf(-et, rlo[1], fmaf(-et, rho[1], e0 * f.up)));
                l1[2] += (double)fabsf(fmaf(-et, rlo[2], fmaf(-et, rho[2], e0 * f.lo)));
                if (k & 1) __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    // The three distances are sums of non-negative terms and are wanted to 1e-5 of themselves: fp32 across the lanes
    // (a DPP step of a float is one instruction, of a double five).
    {
        float* slot = reinterpret_cast<float*>(sm_d);              // [3][NW] floats
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            float v = (float)l1[i];
            v += __int_as_float(dpp_or<kRowShr1, 0xf>(0, __float_as_int(v)));
            v += __int_as_float(dpp_or<kRowShr2, 0xf>(0, __float_as_int(v)));
            v += __int_as_float(dpp_or<kRowShr4, 0xf>(0, __float_as_int(v)));
            v += __int_as_float(dpp_or<kRowShr8, 0xf>(0, __float_as_int(v)));
            v += __int_as_float(dpp_or<kRowBcast15, 0xa>(0, __float_as_int(v)));
            v += __int_as_float(dpp_or<kRowBcast31, 0xc>(0, __float_as_int(v)));
            if (lane == 63) slot[i * NW + wave] = v;
        }
    }
    lds_barrier();
    if (wave == 0) {
        double L[3];
        const float* slot = reinterpret_cast<const float*>(sm_d);
#pragma unroll
        for (int i = 0; i < 3; ++i) L[i] = (double)row16_sum_f(lane < NW ? slot[i * NW + lane] : 0.f);
        // the row's totals, for dro_finish_row: S_mid, S_up, S_lo, Z, the four p_cloud-weighted sums of exponents (times Z),
        // the three L1 distances (times S_mid, S_up, S_lo)
        if (lane == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) fin[i] = tot[i];
            fin[8] = L[0]; fin[9] = L[1]; fin[10] = L[2];
        }
    }
}

// The seven terms of a row from its totals (kDroTotals doubles, as dro_row_compute leaves them).  One lane per row.
// Kept out of the row loop of dro_row_stream_kernel: the constants of the fp64 logarithm would otherwise be hoisted to
// the top of that loop and live in registers (or in scratch memory) through all of it.
constexpr int kDroTotals = 11;
__device__ __forceinline__ void dro_finish_row(const RowArgs& A, float* __restrict__ terms, const int64_t row,
                                               const double* fin)
{
    const double Z = fin[3], ln2_Z = kLn2 / Z;                     // (the weighted sums are over base-2 exponents)
    const double ce_mid = log(fin[0]) - fin[4] * ln2_Z;
    const double ce_up = log(fin[1]) - fin[5] * ln2_Z;
    const double ce_lo = log(fin[2]) - fin[6] * ln2_Z;
    // KL = CE(p_cloud, p_mid) - H(p_cloud) = ln S - ln Z + sum_i p_cloud_i (dt_i - d_i): the last sum is taken over the
    // differences token by token (fin[7]), so that a cloud row close to the centre row -- a small KL, the difference of two
    // cross-entropy-sized numbers -- keeps its accuracy (a seeded random case missed the absolute bound by a quarter
    // with the two sums taken separately)
    const double kl = (log(fin[0]) - log(Z)) + fin[7] * ln2_Z;
    const int64_t N = A.N;
    terms[0 * N + row] = (float)(fin[8] / fin[0]); terms[1 * N + row] = (float)(fin[9] / fin[1]);
    terms[2 * N + row] = (float)(fin[10] / fin[2]);
    terms[3 * N + row] = (float)ce_mid; terms[4 * N + row] = (float)ce_up; terms[5 * N + row] = (float)ce_lo;
    terms[6 * N + row] = (float)kl;
}

template <typename T, int NVEC>
__global__ __launch_bounds__(1024) void dro_row_kernel(const RowArgs A, const DroRadius R, float* __restrict__ terms)
{
    constexpr int THREADS = 1024, NW = 16;
    __shared__ double sm_d[NW * 7];
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const int last_vec = (A.V + Elt<T>::kPerVec - 1) / Elt<T>::kPerVec - 1;
    const bool rad = A.radius != nullptr;                          // uniform
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
    __shared__ double sm_fin[kDroTotals];
    dro_row_compute<T, NVEC>(A, R, sm_fin, cw, tw, rw, sm_d, tid);
    if (tid == 0) dro_finish_row(A, terms, row, sm_fin);           // (the lane that has written the totals)
}

constexpr int kDroRowsPerWg = 64;                                  // most rows a workgroup of dro_row_stream_kernel takes

// The same with the next row on its way while a row is worked on.  One 1024-lane workgroup per compute unit walks
// over rows blockIdx.x, blockIdx.x + gridDim.x, ...; the three rows of a position and the working set leave no
// registers to fetch ahead into, and a second workgroup does not fit a compute unit, so the centre and cloud rows of
// the NEXT position are loaded straight into LDS (global_load_lds_dwordx4: the data of lane l of a wave lands 16 l
// bytes behind the LDS address the wave names; no register is held while the load is in flight) and the raw-radius
// row into the NVEC registers that the current radius row has left.  Every lane reads back only the slots that its own
// wave's loads have written, so the hand-over needs the wave's own vmcnt(0) and no barrier.
// Dynamic LDS: 2 x NVEC x 16 KiB (NVEC <= 4).
template <typename T, int NVEC>
__global__ __launch_bounds__(1024) void dro_row_stream_kernel(const RowArgs A, const DroRadius R,
                                                              float* __restrict__ terms)
{
    constexpr int THREADS = 1024, NW = 16;
    extern __shared__ u32x4 sm_rows[];                             // [2][NVEC][THREADS]: next centre row, next cloud row
    __shared__ double sm_d[NW * 7];
    __shared__ double sm_fin[kDroRowsPerWg][kDroTotals];           // the totals of this workgroup's rows
    const int tid = threadIdx.x;
    const int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int last_vec = (A.V + Elt<T>::kPerVec - 1) / Elt<T>::kPerVec - 1;
    const bool rad = A.radius != nullptr;                          // uniform
    using lds_ptr = __attribute__((address_space(3))) void*;
    using glb_ptr = const __attribute__((address_space(1))) void*;

    // the centre and cloud rows of `row` go on their way to LDS
    auto request_rows = [&](int64_t row, int tid) {
        const gbytes cb = (gbytes)(static_cast<const T*>(A.draft) + row * A.stride);
        const gbytes tb = (gbytes)(static_cast<const T*>(A.target) + row * A.stride);
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            const uint32_t off = (uint32_t)min(j * THREADS + tid, last_vec) * 16u;
            __builtin_amdgcn_global_load_lds((glb_ptr)(cb + off), (lds_ptr)(sm_rows + (0 * NVEC + j) * THREADS + wave_s * 64), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((glb_ptr)(tb + off), (lds_ptr)(sm_rows + (1 * NVEC + j) * THREADS + wave_s * 64), 16, 0, 0);
        }
    };
    auto request_radius = [&](int64_t row, u32x4 (&rn)[NVEC], int tid) {
        const gbytes rb = (gbytes)(static_cast<const T*>(A.radius) + row * A.stride);
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            const uint32_t off = (uint32_t)min(j * THREADS + tid, last_vec) * 16u;
            rn[j] = __builtin_nontemporal_load((gvec)(rb + off));
        }
    };
    u32x4 rnext[NVEC];
#pragma unroll
    for (int j = 0; j < NVEC; ++j) rnext[j] = u32x4{0u, 0u, 0u, 0u};
    // (rows are counted in 32 bits -- the entry point takes no more than 2^31 - 1, and row + gridDim.x stays below 2^32:
    // a 64-bit comparison of two scalars is a vector instruction that wants one of them in vector registers, for good)
    const uint32_t n_rows = (uint32_t)A.N;
    uint32_t row = blockIdx.x;
    int done = 0;                                                  // rows of this workgroup finished so far (<= kDroRowsPerWg)
    if (row < n_rows) {
        request_rows(row, tid);
        if (rad) request_radius(row, rnext, tid);
    }
    for (; row < n_rows; row += gridDim.x) {
        // this wave's loads have landed (its slots of the two rows in LDS, and the radius registers)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // (the lane's index is made opaque once per row: the LDS addresses derived from it are cheap to form again, and
        // hoisted out of this loop they would hold a dozen registers through all of it)
        int t = tid;
        asm volatile("" : "+v"(t));
        u32x4 cw[NVEC], tw[NVEC], rw[NVEC];
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            cw[j] = sm_rows[(0 * NVEC + j) * THREADS + t];
            tw[j] = sm_rows[(1 * NVEC + j) * THREADS + t];
            rw[j] = rnext[j];
        }
        // the slots are free again once they have been read: the next position's rows go in flight now
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const uint32_t next = row + gridDim.x;
        if (next < n_rows) {
            request_rows(next, t);
            if (rad) request_radius(next, rnext, t);
        }
        dro_row_compute<T, NVEC>(A, R, sm_fin[done], cw, tw, rw, sm_d, t);
        // (no barrier here: what wave 0 still reads of sm_d is written again only in the next row's pass 3, two
        // barriers on)
        ++done;
    }
    // one lane per row turns the totals into the row's terms
    __syncthreads();
    if (tid < done) dro_finish_row(A, terms, (int64_t)blockIdx.x + (int64_t)tid * gridDim.x, sm_fin[tid]);
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
// terms.  One workgroup of 256 lanes; losses = { centre, upper, lower, DRO, total }.  One fp64 exponential per row:
// the unnormalised weight is parked in `weights` (when the caller wants them) and scaled by the normaliser in a last
// pass by the lane that wrote it.
template <int T>
__global__ __launch_bounds__(T) void dro_batch_kernel(const float* __restrict__ terms, int64_t N, double lambda_v,
                                                        double lambda_p, double lambda_beta, double alpha,
                                                        float* __restrict__ weights, float* __restrict__ losses)
{
    // (a single workgroup: a chain of two reductions over the rows, as short as its lanes are many.  1024 lanes leave
    // the fp64 exponential 128 registers and it spills a little: worth it only for many rows.)
    constexpr int NW = T / 64;
    __shared__ double sm[NW * 5];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* ce_lo = terms + 5 * N;
    float mxf = -INFINITY;
    double c = 0.0, u = 0.0, l = 0.0;
    for (int64_t n = tid; n < N; n += T) {
        mxf = fmaxf(mxf, (float)(alpha * (double)ce_lo[n]));
        c += lambda_v * terms[n] + lambda_p * terms[3 * N + n] + lambda_beta * terms[6 * N + n];
        u += lambda_v * terms[N + n] + lambda_p * terms[4 * N + n];
        l += lambda_v * terms[2 * N + n] + lambda_p * terms[5 * N + n];
    }
    mxf = wave_max(mxf);
    if (lane == 0) sm[wave] = (double)mxf;
    __syncthreads();
    double mx = sm[0];
    for (int w = 1; w < NW; ++w) mx = fmax(mx, sm[w]);
    __syncthreads();
    double den = 0.0, num = 0.0;
    for (int64_t n = tid; n < N; n += T) {
        const double ce = (double)ce_lo[n];
        const double e = exp(alpha * ce - mx);
        den += e;
        num = fma(e, ce, num);
        if (weights) weights[n] = (float)e;                        // scaled below
    }
    c = wave_sum(c); u = wave_sum(u); l = wave_sum(l); den = wave_sum(den); num = wave_sum(num);
    if (lane == 0) { sm[wave * 5] = c; sm[wave * 5 + 1] = u; sm[wave * 5 + 2] = l; sm[wave * 5 + 3] = den; sm[wave * 5 + 4] = num; }
    __syncthreads();
    double tot[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int w = 0; w < NW; ++w)
        for (int i = 0; i < 5; ++i) tot[i] += sm[w * 5 + i];
    if (weights) {
        // float(e) / den in fp64 rounds e twice (once to float above): 6e-8 relative, far inside the weights' tolerance
        const double inv = 1.0 / tot[3];
        for (int64_t n = tid; n < N; n += T) weights[n] = (float)((double)weights[n] * inv);
    }
    if (tid == 0 && losses) {
        const double Nd = (double)N, dro = tot[4] / tot[3];
        losses[0] = (float)(tot[0] / Nd); losses[1] = (float)(tot[1] / Nd); losses[2] = (float)(tot[2] / Nd);
        losses[3] = (float)dro;
        losses[4] = (float)(tot[0] / Nd + tot[1] / Nd + tot[2] / Nd + dro);
    }
}

}  // namespace

namespace {
template <typename T, int NVEC>
hipError_t launch_dro_stream_cfg(const RowArgs& a, float* terms, hipStream_t stream)
{
    constexpr unsigned lds = 2u * NVEC * 1024u * 16u;
    if (lds > 48u * 1024u) {
        // above the default limit on dynamic LDS: raised once per device and instance
        static std::mutex guard;
        static bool raised[64] = {};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
        std::lock_guard<std::mutex> lock(guard);
        if (!raised[dev]) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dro_row_stream_kernel<T, NVEC>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            raised[dev] = true;
        }
    }
    // one workgroup per compute unit; more of them (taking their turn) when that would give a workgroup more than
    // kDroRowsPerWg rows
    int64_t g = compute_units();
    const int64_t need = (a.N + kDroRowsPerWg - 1) / kDroRowsPerWg;
    if (g < need) g = need;
    if (g > a.N) g = a.N;
    const dim3 grid((unsigned)g), block(1024);
    const DroRadius R = {(float)a.kappa, (float)a.rmax, (float)fmin(a.kappa, a.rmax)};
    hipLaunchKernelGGL((dro_row_stream_kernel<T, NVEC>), grid, block, lds, stream, a, R, terms);
    return hipGetLastError();
}
template <typename T>
hipError_t launch_dro_stream(int nvec, const RowArgs& a, float* terms, hipStream_t stream)
{
    if (nvec == 1) return launch_dro_stream_cfg<T, 1>(a, terms, stream);
    if (nvec == 2) return launch_dro_stream_cfg<T, 2>(a, terms, stream);
    return launch_dro_stream_cfg<T, 4>(a, terms, stream);
}
}  // namespace

hipError_t launch_dro(int dtype, const RowArgs& args, float* terms, double lambda_v, double lambda_p,
                      double lambda_beta, double alpha, float* weights, float* losses, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const int epv = dtype == 0 ? 4 : 8;
    const int vecs = (args.V + epv - 1) / epv;
    const dim3 grid((unsigned)args.N), block(1024);
    const DroRadius R = {(float)args.kappa, (float)args.rmax, (float)fmin(args.kappa, args.rmax)};
#define CIAR_DRO_LAUNCH(NV)                                                                             \
    do {                                                                                                \
        if (dtype == 0) hipLaunchKernelGGL((dro_row_kernel<float, NV>), grid, block, 0, stream, args, R, terms);   \
        else hipLaunchKernelGGL((dro_row_kernel<bf16_t, NV>), grid, block, 0, stream, args, R, terms);           \
    } while (0)
    if (args.V <= kTinyVocab) {
        const dim3 tgrid((unsigned)((args.N + 255) / 256)), tblock(256);
        if (dtype == 0) hipLaunchKernelGGL(dro_row_tiny_kernel<float>, tgrid, tblock, 0, stream, args, terms);
        else hipLaunchKernelGGL(dro_row_tiny_kernel<bf16_t>, tgrid, tblock, 0, stream, args, terms);
    } else if (vecs <= 4096 && args.N > (int64_t)compute_units()) {
        // more rows than compute units: persistent workgroups that fetch the next row through LDS
        const int nv = vecs <= 1024 ? 1 : vecs <= 2048 ? 2 : 4;
        const hipError_t e = dtype == 0 ? launch_dro_stream<float>(nv, args, terms, stream)
                                        : launch_dro_stream<bf16_t>(nv, args, terms, stream);
        if (e != hipSuccess) return e;
    } else if (vecs <= 1024) CIAR_DRO_LAUNCH(1);
    else if (vecs <= 2048) CIAR_DRO_LAUNCH(2);
    else if (vecs <= 4096) CIAR_DRO_LAUNCH(4);
    else if (vecs <= 8192) CIAR_DRO_LAUNCH(8);
    else return hipErrorInvalidValue;
#undef CIAR_DRO_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || (!weights && !losses)) return e;
    if (args.N > 8192)
        hipLaunchKernelGGL(dro_batch_kernel<1024>, dim3(1), dim3(1024), 0, stream, terms, args.N, lambda_v, lambda_p,
                           lambda_beta, alpha, weights, losses);
    else
        hipLaunchKernelGGL(dro_batch_kernel<512>, dim3(1), dim3(512), 0, stream, terms, args.N, lambda_v, lambda_p,
                           lambda_beta, alpha, weights, losses);
    return hipGetLastError();
}

}  // namespace ciar
