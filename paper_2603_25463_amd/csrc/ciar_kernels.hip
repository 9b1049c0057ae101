// gfx950 kernels of the CIAR quantify + verify pass.
//
// The pass is split so that the kernel that touches the V-wide rows is pure streaming arithmetic:
//
//   stream_kernel   reads every logit row exactly once from HBM and leaves ten numbers per row
//                   (RowStats).  A workgroup of 256 lanes (512 or 1024 for large vocabularies or few
//                   rows) owns one row at a time and walks over rows blockIdx.x, blockIdx.x +
//                   gridDim.x, ...  The grid is exactly the workgroups that are resident at once (four
//                   waves per SIMD): while one workgroup waits for its row, the others compute, which
//                   keeps the memory system busy without a second set of row registers.  Loads are
//                   interleaved over the workgroup so that every load instruction of a wave covers
//                   1 KiB of consecutive memory.  Nothing V-wide is ever written back.
//   rowfinish_kernel  one thread per row turns RowStats into the row's outputs in fp64 (caps, Omega,
//                   Sigma, U, flag, interval of the reported token, accept test) and appends rejected
//                   rows to a list.
//   resample_kernel 1024-lane workgroups walk over that list (~1 row in 8) and run the residual draw,
//                   re-reading the two rows (mostly served by the caches).
//
// The centre row has to be resident between its statistics pass and its interval pass: the InterFuse
// bounds need the partition sum S of the complete row before the first bound can be formed (App.
// "Proof of Interval Validity": S appears in every denominator).  It lives in registers as
// e_i = 2^(c_i log2e - n_w).  The verifier row is only needed for max / Z and is consumed on arrival.
//
// stream_kernel, per row (centre row first: it carries most of the arithmetic, so that little is left
// to do when the last bytes of a launch arrive):
//   B  centre row:   per-wave maximum, e_i = 2^(c_i log2e - n_w) kept in registers, S_w = sum e_i
//      The reference n_w is an integer (the next integer above max * log2e of the *wave*), so the
//      waves need no barrier before exponentiating and their results combine exactly:
//      S = sum_w S_w 2^(n_w - n), n = max_w n_w, a power-of-two rescale.
//   -- barrier: the waves exchange (max, n_w, S_w) --
//   C  InterFuse for a scalar radius r, a = e^r, b = e^-r, x_i = e_i / S:
//        p^u_i = a x_i / (1 + (a-1) x_i),   p^l_i = b x_i / (1 - (1-b) x_i)
//      with one reciprocal of the product of the two denominators, accumulated as the lower
//      bound p^l_i and the raw width w_i = p^u_i - p^l_i = (a-b) x_i (1-x_i) / (du_i dl_i):
//      five fp64 sums per row (sum p^l, sum w and the three second moments); two of them when the
//      row's largest probability shows that the caps cannot be active.
//   T  verifier row, loaded into the registers the centre row came in: per-wave maximum,
//      Z_w = sum 2^(t_i log2e - nt_w)                                               (max-trick)
//   -- barrier: the waves exchange their interval sums and (nt_w, Z_w); thread 0 writes RowStats --
//
// rowfinish_kernel / resample_kernel, per row (Eq. uncertainty_score; Algorithm 1's threshold and verification steps):
//   delta_i = alpha_u w_i + (alpha_u - alpha_l) p^l_i once the 0.99 / 1.01 caps alpha_l, alpha_u are
//   known, so Omega = sum delta_i, Sigma^2 = (sum delta_i^2) / V - (Omega / V)^2, U = Omega * Sigma
//   follow from the five sums without a second sweep over the row; flag = U > tau;
//   accept iff ln u < min(0, ln q_x - ln p_x) (log domain, fp64);
//   rejected rows: res_i = max(0, q_i - p_i), inverse-CDF draw in token order from a workgroup-wide
//   prefix sum.
//
// Sums over a row are accumulated per lane (S and the five interval sums in fp64, which this chip
// issues at the fp32 rate) and combined across lanes with DPP and across waves through LDS in a fixed
// order, so results are deterministic and the per-row scalars carry ~1e-8 relative error.
#include "ciar_internal.h"

#include <limits.h>
#include <math.h>

namespace ciar {
namespace {

// log2(e) split so that the low part is positive: x * hi + x * lo stays -inf for x = -inf.
constexpr float  kLog2eHi = 1.44269490242004394531f;   // largest float below log2(e)
constexpr float  kLog2eLo = 1.384689195e-7f;           // log2(e) - kLog2eHi
constexpr double kLn2 = 0.69314718055994530942;

__device__ __forceinline__ float bits_f(uint32_t u) { return __uint_as_float(u); }

// 16 bytes as loaded: a native vector type, so it can be read through an address-space pointer.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
using gbytes = const __attribute__((address_space(1))) char*;
using gvec = const __attribute__((address_space(1))) u32x4*;

// 2^(x log2(e) - n) for an integer-valued reference n.  x * hi - n is exact inside the FMA and is
// rounded at the magnitude of the (small) result; the low part of log2(e) is added by a second FMA.
__device__ __forceinline__ float exp2_ref(float x, float n)
{
    return __builtin_amdgcn_exp2f(fmaf(x, kLog2eLo, fmaf(x, kLog2eHi, -n)));
}

// Integer reference for a set of logits whose maximum is m: the next integer above m * log2(e), so
// every 2^(x log2e - n) is <= 1 (up to rounding).  -inf (nothing but masked tokens) maps to -inf.
__device__ __forceinline__ float ref_of(float m) { return ceilf(m * 1.44269504f); }

// 2^k as a double for an integer-valued float difference k <= 0 (clamped: below 2^-1000 it is 0 anyway)
__device__ __forceinline__ double pow2_of(float k) { return ldexp(1.0, (int)fmaxf(k, -1000.f)); }

template <typename T> struct Elt;
template <> struct Elt<float> {
    static constexpr int kPerVec = 4;
    static constexpr uint32_t kNegInfWord = 0xff800000u;
    __device__ static __forceinline__ void unpack(const u32x4& r, float* o)
    {
        o[0] = bits_f(r.x); o[1] = bits_f(r.y); o[2] = bits_f(r.z); o[3] = bits_f(r.w);
    }
    // Replace elements with index >= V of a vector that starts at element `base` by -inf.
    __device__ static __forceinline__ void mask_tail(u32x4& r, int base, int V)
    {
        if (base + 0 >= V) r.x = kNegInfWord;
        if (base + 1 >= V) r.y = kNegInfWord;
        if (base + 2 >= V) r.z = kNegInfWord;
        if (base + 3 >= V) r.w = kNegInfWord;
    }
    // ... by zero.
    __device__ static __forceinline__ void zero_tail(u32x4& r, int base, int V)
    {
        if (base + 0 >= V) r.x = 0u;
        if (base + 1 >= V) r.y = 0u;
        if (base + 2 >= V) r.z = 0u;
        if (base + 3 >= V) r.w = 0u;
    }
};
struct bf16_t { uint16_t bits; };
template <> struct Elt<bf16_t> {
    static constexpr int kPerVec = 8;
    static constexpr uint32_t kNegInfWord = 0xff80ff80u;
    __device__ static __forceinline__ void unpack(const u32x4& r, float* o)
    {
        o[0] = bits_f(r.x << 16); o[1] = bits_f(r.x & 0xffff0000u);
        o[2] = bits_f(r.y << 16); o[3] = bits_f(r.y & 0xffff0000u);
        o[4] = bits_f(r.z << 16); o[5] = bits_f(r.z & 0xffff0000u);
        o[6] = bits_f(r.w << 16); o[7] = bits_f(r.w & 0xffff0000u);
    }
    __device__ static __forceinline__ uint32_t mask_word(uint32_t w, int base, int V)
    {
        if (base >= V) return kNegInfWord;
        if (base + 1 >= V) return (w & 0x0000ffffu) | 0xff800000u;
        return w;
    }
    __device__ static __forceinline__ void mask_tail(u32x4& r, int base, int V)
    {
        r.x = mask_word(r.x, base + 0, V); r.y = mask_word(r.y, base + 2, V);
        r.z = mask_word(r.z, base + 4, V); r.w = mask_word(r.w, base + 6, V);
    }
    __device__ static __forceinline__ uint32_t zero_word(uint32_t w, int base, int V)
    {
        return w & ((base < V ? 0x0000ffffu : 0u) | (base + 1 < V ? 0xffff0000u : 0u));
    }
    __device__ static __forceinline__ void zero_tail(u32x4& r, int base, int V)
    {
        r.x = zero_word(r.x, base + 0, V); r.y = zero_word(r.y, base + 2, V);
        r.z = zero_word(r.z, base + 4, V); r.w = zero_word(r.w, base + 6, V);
    }
};

template <typename T>
__device__ __forceinline__ float load_logit(const T* row, int i)
{
    if constexpr (sizeof(T) == 4) return reinterpret_cast<const float*>(row)[i];
    else return bits_f((uint32_t)reinterpret_cast<const uint16_t*>(row)[i] << 16);
}

// ---- wave reductions (fixed order: deterministic) ----------------------------------------------
//
// DPP row shifts and row broadcasts: they run on the vector ALU at full rate, whereas a shuffle
// (ds_bpermute) goes through the LDS crossbar and costs ~5x more per step.
// Pattern (wave64 = 4 rows of 16 lanes): row_shr 1, 2, 4, 8 leave each row's inclusive prefix in its
// lanes; row_bcast:15 adds a row's total into the next row (rows 1 and 3), row_bcast:31 adds lane 31
// into rows 2 and 3; every lane then holds its inclusive prefix over the wave and lane 63 the total,
// which readlane hands to every lane.

constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;

// value of the lane selected by CTRL, or `fill` where the selection is out of range / masked off
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_or(int fill, int v)
{
    return __builtin_amdgcn_update_dpp(fill, v, CTRL, ROW_MASK, 0xf, false);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add(double v)
{
    const int lo = dpp_or<CTRL, ROW_MASK>(0, __double2loint(v));
    const int hi = dpp_or<CTRL, ROW_MASK>(0, __double2hiint(v));
    return v + __hiloint2double(hi, lo);           // lanes without a source add +0.0
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ double wave_scan(double v)
{
    v = dpp_add<kRowShr1, 0xf>(v);
    v = dpp_add<kRowShr2, 0xf>(v);
    v = dpp_add<kRowShr4, 0xf>(v);
    v = dpp_add<kRowShr8, 0xf>(v);
    v = dpp_add<kRowBcast15, 0xa>(v);
    v = dpp_add<kRowBcast31, 0xc>(v);
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
    v = wave_scan(v);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max(float v)
{
    // lanes without a source get their own value back: max(v, v) = v
    return fmaxf(v, __int_as_float(dpp_or<CTRL, ROW_MASK>(__float_as_int(v), __float_as_int(v))));
}

__device__ __forceinline__ float wave_max(float v)
{
    v = dpp_max<kRowShr1, 0xf>(v);
    v = dpp_max<kRowShr2, 0xf>(v);
    v = dpp_max<kRowShr4, 0xf>(v);
    v = dpp_max<kRowShr8, 0xf>(v);
    v = dpp_max<kRowBcast15, 0xa>(v);
    v = dpp_max<kRowBcast31, 0xc>(v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ int wave_min_i(int v)
{
    v = min(v, dpp_or<kRowShr1, 0xf>(v, v));
    v = min(v, dpp_or<kRowShr2, 0xf>(v, v));
    v = min(v, dpp_or<kRowShr4, 0xf>(v, v));
    v = min(v, dpp_or<kRowShr8, 0xf>(v, v));
    v = min(v, dpp_or<kRowBcast15, 0xa>(v, v));
    v = min(v, dpp_or<kRowBcast31, 0xc>(v, v));
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ int wave_max_i(int v)
{
    v = max(v, dpp_or<kRowShr1, 0xf>(v, v));
    v = max(v, dpp_or<kRowShr2, 0xf>(v, v));
    v = max(v, dpp_or<kRowShr4, 0xf>(v, v));
    v = max(v, dpp_or<kRowShr8, 0xf>(v, v));
    v = max(v, dpp_or<kRowBcast15, 0xa>(v, v));
    v = max(v, dpp_or<kRowBcast31, 0xc>(v, v));
    return __builtin_amdgcn_readlane(v, 63);
}

// ---- per-token InterFuse arithmetic, shared by the streaming kernel and the dense export ------------

// Constants of one row for a scalar radius.  Units: e_i as held by the lane, S = sum e_i in the same units.
struct FuseRow {
    float cu;            // (a-1)/S:  du = 1 + (a-1) x = 1 + cu e
    float nih, nil;      // -1/S split in two floats:  1 - x = 1 + nih e + nil e  (exact to ~1e-15)
    float b, omb;        // b and 1-b:  dl = 1 - (1-b) x = b + (1-b)(1-x), free of cancellation as x -> 1
};

__device__ __forceinline__ FuseRow fuse_row(double S, double a, double b)
{
    FuseRow r;
    const double invS = 1.0 / S;
    r.cu = (float)((a - 1.0) * invS);
    r.nih = (float)(-invS);
    r.nil = (float)(-invS - (double)r.nih);
    r.b = (float)b;
    r.omb = (float)(1.0 - b);
    return r;
}

// gl = e du / (du dl) and gw = e (1-x) / (du dl):  p^l = (b/S) gl,  w = p^u - p^l = ((a-b)/S) gw.
// SPLIT = form 1 - x with the two-float 1/S.  It matters only when some x is close to 1 (the relative
// error of 1 - x is 6e-8 x / (1 - x) without it); rows whose largest probability is at most 1/2 skip it.
template <bool SPLIT = true>
__device__ __forceinline__ void fuse_token(float e, const FuseRow& r, float& gl, float& gw)
{
    const float om = SPLIT ? fmaf(e, r.nil, fmaf(e, r.nih, 1.0f)) : fmaf(e, r.nih, 1.0f);   // 1 - x
    const float du = fmaf(e, r.cu, 1.0f);
    const float dl = fmaf(om, r.omb, r.b);
    const float g = e * __builtin_amdgcn_rcpf(du * dl);
    gl = g * du;
    gw = g * om;
}

// Tensor-radius mode (Sec. 3.2.3, the Interval Head: r = Softplus(raw)): a = e^r, b = e^-r for
// r = min(kappa Softplus(raw), rmax).  Softplus(raw) = max(raw, 0) + ln(1 + t), t = e^-|raw|;
// ln(1 + t) = ln(u) t / (u - 1) with u = fl(1 + t): u - 1 is exact, so the rounding of 1 + t cancels in
// the ratio and small radii (raw << 0) keep their relative accuracy.
__device__ __forceinline__ void radius_ab(float raw, float kappa, float rmax, float& a, float& b)
{
    const float t = __builtin_amdgcn_exp2f(-fabsf(raw) * 1.44269504f);
    const float u = 1.0f + t;
    const float d = u - 1.0f;
    const float lg = d == 0.f ? t : (__builtin_amdgcn_logf(u) * 0.693147181f) * (t * __builtin_amdgcn_rcpf(d));
    const float r = fminf(kappa * (fmaxf(raw, 0.f) + lg), rmax);
    a = __builtin_amdgcn_exp2f(r * 1.44269504f);
    b = __builtin_amdgcn_rcpf(a);
}

// The same radius in fp64 (one token per row: the reported token's interval).
__device__ __forceinline__ double radius_of(double raw, double kappa, double rmax)
{
    const double sp = raw > 0.0 ? raw + log1p(exp(-raw)) : log1p(exp(raw));
    return fmin(kappa * sp, rmax);
}

// Tensor-radius token: pl = p^l_i S and w = (p^u_i - p^l_i) S in the units of e.
__device__ __forceinline__ void fuse_token_rad(float e, float raw, const FuseRow& r, float kappa, float rmax,
                                               float& pl, float& w)
{
    float a, b;
    radius_ab(raw, kappa, rmax, a, b);
    const float om = fmaf(e, r.nil, fmaf(e, r.nih, 1.0f));        // 1 - x
    const float x = -e * r.nih;
    const float du = fmaf(a - 1.0f, x, 1.0f);
    const float dl = fmaf(om, 1.0f - b, b);
    const float g = e * __builtin_amdgcn_rcpf(du * dl);
    pl = b * (g * du);
    w = (a - b) * (g * om);
}

// Per-row scalars of the quantifier from the five sums (fp64, one lane).
struct RowScore { double alpha_l, alpha_u, omega, sigma, score; };

__device__ __forceinline__ RowScore finish_score(const double* s, double S, bool capless, const RowArgs& A)
{
    // s = { sum gl, sum gw, sum gl^2, sum gw^2, sum gl gw } over the V tokens of the row, with
    // p^l_i = Bc gl_i and p^u_i - p^l_i = Wc gw_i (tensor-radius mode: the per-token factors are already
    // inside gl and gw);
    // capless = the caps are known to be inactive and only sum gw, sum gw^2 were accumulated
    const double V = (double)A.V;
    const double Bc = (A.radius ? 1.0 : A.b) / S, Wc = (A.radius ? 1.0 : A.a - A.b) / S;
    const double Sl = Bc * s[0], Su = Sl + Wc * s[1];
    RowScore o;
    o.alpha_l = 1.0; o.alpha_u = 1.0;
    if (A.normalize && !capless) {
        o.alpha_l = fmin(1.0, A.cap_lo / Sl);
        o.alpha_u = fmax(1.0, A.cap_hi / Su);
    }
    // delta_i = alpha_u p^u_i - alpha_l p^l_i = alpha_u w_i + (alpha_u - alpha_l) p^l_i = cw gw_i + cl gl_i:
    // both coefficients are >= 0, so Omega and the second moment are sums of non-negative terms.
    const double cw = o.alpha_u * Wc, cl = (o.alpha_u - o.alpha_l) * Bc;
    o.omega = cw * s[1] + cl * s[0];
    const double Q = cw * cw * s[3] + 2.0 * cw * cl * s[4] + cl * cl * s[2];
    // fp64 sums: the subtraction of the squared mean costs at most ~1/CV^2 of 1e-16
    const double var = fmax(0.0, Q - o.omega * o.omega / V) / V;
    o.sigma = sqrt(var);
    o.score = o.omega * o.sigma;
    return o;
}

// ---- the streaming kernel ---------------------------------------------------------------------------------

// Waves per SIMD the register allocation aims for: the centre row held as floats plus ~40 working
// registers, capped at 4 waves.  Memory latency is hidden by the other resident workgroups of the compute
// unit rather than by fetching ahead into a second set of registers: measured on this chip, three or
// four resident workgroups beat two with a register prefetch of the next row at every vocabulary size.
// (Tensor-radius mode: the raw radius row sits in registers next to the centre row during the interval pass.)
template <typename T, int THREADS, int NVEC, bool RAD>
constexpr int target_waves()
{
    constexpr int ept = NVEC * Elt<T>::kPerVec;                    // one row as floats
    constexpr int fit = 512 / (ept + (RAD ? NVEC * 4 + 8 : 0) + 40);
    constexpr int lo = THREADS / 256;                              // waves per SIMD one workgroup needs
    return fit < lo ? lo : (fit > 4 ? 4 : fit);
}

// Pass C for one lane: the InterFuse sums over the lane's tokens.
// Chunks past the end of a row that does not fill the tile are skipped (padding inside the last chunk
// has e = 0 and adds exactly nothing).
// WIDTH_ONLY = the caps are known to be inactive for this row (alpha_l = alpha_u = 1), so
// delta_i = w_i and only sum gw and sum gw^2 are needed.
// SPLIT = see fuse_token.
template <int THREADS, int NVEC, int EPV, bool WIDTH_ONLY, bool SPLIT>
__device__ __forceinline__ void fuse_sums(const float (&e)[NVEC * EPV], const FuseRow& fr, int V,
                                          double (&q5)[5])
{
    // The sums run in fp64 from the first add (fp64 adds and FMAs issue at the fp32 rate on this
    // chip).  One token can hold almost all of sum(gl), and the variance is a difference of second
    // moments that would cancel in fp32 on nearly flat rows; in fp64 neither needs a centring trick.
    double a0[2] = {0.0, 0.0}, a1[2] = {0.0, 0.0}, a2[2] = {0.0, 0.0}, a3[2] = {0.0, 0.0}, a4[2] = {0.0, 0.0};
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        if (j * THREADS * EPV >= V) continue;                      // uniform: the chunk holds no token
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float gl, gw;
            fuse_token<SPLIT>(e[j * EPV + k], fr, gl, gw);         // padding has e = 0: gl = gw = 0
            const double dw = (double)gw;
            a1[k & 1] += dw;
            a3[k & 1] = fma(dw, dw, a3[k & 1]);
            if constexpr (!WIDTH_ONLY) {
                const double dl = (double)gl;
                a0[k & 1] += dl;
                a2[k & 1] = fma(dl, dl, a2[k & 1]);
                a4[k & 1] = fma(dl, dw, a4[k & 1]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);                         // one vector at a time: bounded working set
    }
    q5[0] = a0[0] + a0[1];
    q5[1] = a1[0] + a1[1];
    q5[2] = a2[0] + a2[1];
    q5[3] = a3[0] + a3[1];
    q5[4] = a4[0] + a4[1];
}

// Pass C for a handful of tokens (V <= kTinyVocab), in fp64 from the fp32 e_i.  With so few tokens the widths
// are O(1) and Sigma can be an exact zero (two tokens: delta_1 = delta_2 identically, because x_1 + x_2 = 1
// holds for the computed x as well); fp32 token arithmetic leaves ~1e-7 there, fp64 keeps the symmetry.
// Same units as fuse_sums / fuse_sums_rad: gl, gw per token with p^l = Bc gl, p^u - p^l = Wc gw.
constexpr int kTinyVocab = 64;

template <typename T, int EPV, bool RAD>
__device__ __forceinline__ void fuse_sums_tiny(const float (&e)[EPV], const u32x4& rad, double S_units, double a,
                                               double b, double kappa, double rmax, double (&q5)[5])
{
    float raw[EPV];
    Elt<T>::unpack(rad, raw);
    const double invS = 1.0 / S_units;
#pragma unroll
    for (int i = 0; i < 5; ++i) q5[i] = 0.0;
#pragma unroll
    for (int k = 0; k < EPV; ++k) {
        const double ed = (double)e[k], x = ed * invS;
        double ak = a, bk = b;
        if constexpr (RAD) {
            const double r = radius_of((double)raw[k], kappa, rmax);
            ak = exp(r); bk = exp(-r);
        }
        const double om = 1.0 - x, du = 1.0 + (ak - 1.0) * x, dl = 1.0 - (1.0 - bk) * x;
        double gl = ed / dl, gw = ed * om / (du * dl);
        if constexpr (RAD) { gl *= bk; gw *= ak - bk; }
        q5[0] += gl; q5[1] += gw;
        q5[2] = fma(gl, gl, q5[2]); q5[3] = fma(gw, gw, q5[3]); q5[4] = fma(gl, gw, q5[4]);
    }
}

// Pass C in tensor-radius mode: every token has its own a_i, b_i from the raw radius row `rad` (as loaded,
// padding already zeroed); the sums are of p^l_i S and (p^u_i - p^l_i) S themselves.
template <typename T, int THREADS, int NVEC>
__device__ __forceinline__ void fuse_sums_rad(const float (&e)[NVEC * Elt<T>::kPerVec], const u32x4 (&rad)[NVEC],
                                              const FuseRow& fr, float kappa, float rmax, int V, double (&q5)[5])
{
    constexpr int EPV = Elt<T>::kPerVec;
    double a0[2] = {0.0, 0.0}, a1[2] = {0.0, 0.0}, a2[2] = {0.0, 0.0}, a3[2] = {0.0, 0.0}, a4[2] = {0.0, 0.0};
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        if (j * THREADS * EPV >= V) continue;                      // uniform: the chunk holds no token
        float raw[EPV];
        Elt<T>::unpack(rad[j], raw);
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float pl, w;
            fuse_token_rad(e[j * EPV + k], raw[k], fr, kappa, rmax, pl, w);   // padding has e = 0: pl = w = 0
            const double dl = (double)pl, dw = (double)w;
            a0[k & 1] += dl;
            a1[k & 1] += dw;
            a2[k & 1] = fma(dl, dl, a2[k & 1]);
            a3[k & 1] = fma(dw, dw, a3[k & 1]);
            a4[k & 1] = fma(dl, dw, a4[k & 1]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    q5[0] = a0[0] + a0[1];
    q5[1] = a1[0] + a1[1];
    q5[2] = a2[0] + a2[1];
    q5[3] = a3[0] + a3[1];
    q5[4] = a4[0] + a4[1];
}

template <typename T, int THREADS, int NVEC, bool DO_Q, bool DO_V, bool RAD>
__global__ __launch_bounds__(THREADS)
__attribute__((amdgpu_waves_per_eu(target_waves<T, THREADS, NVEC, RAD>())))
void stream_kernel(const RowArgs A)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec;
    constexpr int EPT = NVEC * EPV;
    constexpr int NW = THREADS / 64;
    constexpr int CHUNK = THREADS * EPV;            // tokens covered by one load instruction of the workgroup

    // Exchange slots.  Two barriers per row order every write against every read: the centre-row
    // slots are written before the first and read between the two, the others are written between the
    // two and read by thread 0 after the second, before it reaches the next row's first barrier.
    __shared__ float  sm_ref[NW * 2];               // per wave: max centre logit, n_w
    __shared__ double sm_S[NW];                     // per wave: S_w
    __shared__ float  sm_nt[NW];                    // per wave: nt_w
    __shared__ double sm_Z[NW];                     // per wave: Z_w
    __shared__ double sm_q5[NW * 5];                // per wave: the five interval sums, already in row units

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = A.V;
    const bool partial = V != NVEC * CHUNK;                        // uniform: the row does not fill the tile
    const int last_vec = (V + EPV - 1) / EPV - 1;
    const int nrows = (int)A.N;
    const int step = (int)gridDim.x;

    // Rows live in global memory (address space 1).  Vector j of this lane: scalar row base + 32-bit
    // byte offset.  A row that fills the tile needs one lane offset for all of its vectors (the
    // distance between vectors is a constant on top of the scalar base).  Otherwise vector indices
    // past the end of the row are clamped to its last vector, so every lane loads valid memory
    // unconditionally; tokens that do not exist are set to -inf afterwards.
    // The base goes through readfirstlane and the lane index through an empty asm: both are opaque
    // to the optimiser, which otherwise turns the sixteen addresses of a row into sixteen 64-bit
    // induction variables, spills them, and serialises the loads on the reloads.
    auto load_row = [&](u32x4 (&buf)[NVEC], const void* rows, int r) {
        const uint64_t b = (uint64_t)(static_cast<const T*>(rows) + (int64_t)r * A.stride);
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
        const gbytes base = (gbytes)(((uint64_t)hi << 32) | lo);
        int t = tid;
        asm volatile("" : "+v"(t));
        if (partial) {
#pragma unroll
            for (int j = 0; j < NVEC; ++j) {
                const uint32_t off = (uint32_t)min(j * THREADS + t, last_vec) * 16u;
                buf[j] = *(gvec)(base + off);
            }
        } else {
            const uint32_t off = (uint32_t)t * 16u;
#pragma unroll
            for (int j = 0; j < NVEC; ++j) buf[j] = *(gvec)(base + (uint64_t)j * (THREADS * 16u) + off);
        }
    };
    // Verifier row statistics of one wave from the row as loaded: nt_w and Z_w = sum 2^(t_i log2e - nt_w).
    auto verifier_stats = [&](u32x4 (&tb)[NVEC], float& ntw, double& Zw) {
        if (partial) {
#pragma unroll
            for (int j = 0; j < NVEC; ++j) E::mask_tail(tb[j], (j * THREADS + tid) * EPV, V);
        }
        float mt = -INFINITY;
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            float tv[EPV];
            E::unpack(tb[j], tv);
#pragma unroll
            for (int k = 0; k < EPV; ++k) mt = fmaxf(mt, tv[k]);
        }
        ntw = ref_of(wave_max(mt));
        const float nref = ntw == -INFINITY ? 0.f : ntw;           // an all-masked wave: every term is 2^-inf = 0
        float zacc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            float tv[EPV];
            E::unpack(tb[j], tv);
#pragma unroll
            for (int k = 0; k < EPV; ++k) zacc[k & 3] += exp2_ref(tv[k], nref);
            __builtin_amdgcn_sched_barrier(0);
        }
        Zw = wave_sum((double)((zacc[0] + zacc[1]) + (zacc[2] + zacc[3])));
    };

    // the list of rejected rows that the finishing kernels build starts empty
    if (DO_V && blockIdx.x == 0 && tid == 0) *A.reject_count = 0;

    // The row index is uniform over the workgroup: keep it in a scalar register.
    // A row's centre logits are loaded and worked on first, its verifier logits second: the centre row
    // carries most of the arithmetic (both of its passes), the verifier row only a short one, so
    // little work is left when the last bytes of the launch arrive.
    int row = __builtin_amdgcn_readfirstlane((int)blockIdx.x);     // the launcher keeps gridDim.x <= N
    u32x4 buf[NVEC];                                               // a row as loaded: centre and verifier row in turn
    load_row(buf, A.draft, row);

    for (;;) {
        const int next = __builtin_amdgcn_readfirstlane(row + step);
        const bool has_next = next < nrows;                        // uniform

        // ---- B: centre row: per-wave max, e_i = 2^(c_i log2e - n_w), S_w -------------------------------
        float e[EPT];
        if (partial) {
#pragma unroll
            for (int j = 0; j < NVEC; ++j) E::mask_tail(buf[j], (j * THREADS + tid) * EPV, V);
        }
#pragma unroll
        for (int j = 0; j < NVEC; ++j) E::unpack(buf[j], &e[j * EPV]);
        float mcl = e[0];
#pragma unroll
        for (int i = 1; i < EPT; ++i) mcl = fmaxf(mcl, e[i]);
        const float mcw = wave_max(mcl);
        const float nw = ref_of(mcw);
        double Sw;
        {
            // S is accumulated in fp64 from the first add: on a nearly one-hot row the bounds of the top
            // token react to a relative error in S about five times over, and on a two-token row Sigma is
            // a difference of two nearly equal widths; even one fp32 add of two comparable terms (6e-8)
            // shows there (measured against the fp64 definition).
            const float nref = nw == -INFINITY ? 0.f : nw;
            double sacc[2] = {0.0, 0.0};
#pragma unroll
            for (int j = 0; j < NVEC; ++j) {
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    e[j * EPV + k] = exp2_ref(e[j * EPV + k], nref);
                    sacc[k & 1] += (double)e[j * EPV + k];
                }
                __builtin_amdgcn_sched_barrier(0);                 // keep the working set to one vector at a time
            }
            Sw = wave_sum(sacc[0] + sacc[1]);
        }

        // ---- the waves exchange the centre row's statistics ----------------------------------------------
        if (lane == 0) {
            sm_ref[wave * 2] = mcw; sm_ref[wave * 2 + 1] = nw;
            sm_S[wave] = Sw;
        }
        __syncthreads();
        float mc = sm_ref[0], n = sm_ref[1];
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            mc = fmaxf(mc, sm_ref[w * 2]);
            n = fmaxf(n, sm_ref[w * 2 + 1]);
        }
        double S = 0.0;                                            // in units of 2^-n
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float rn = sm_ref[w * 2 + 1];
            if (rn != -INFINITY) S += sm_S[w] * pow2_of(rn - n);
        }
        const double fw = nw == -INFINITY ? 0.0 : pow2_of(nw - n);     // this wave's e_i are 1/fw too large

        // ---- C: InterFuse sums in this wave's units, rescaled to row units by lane 0 of the wave ---------
        // Caps: S_l <= b / (1 - (1-b) x_max) and S_u >= a / (1 + (a-1) x_max) for the largest probability
        // x_max of the row, so below the host-computed bound on x_max both caps are inactive and the
        // cheaper width-only pass is exact.  Uniform over the workgroup.
        const double emax = (double)exp2_ref(mc, n);               // the row's largest e_i, in row units
        const bool capless = !A.normalize || (!RAD && emax <= A.capless_xmax * S);
        const bool split = emax > 0.5 * S;                         // some x_i above 1/2: 1 - x needs the two-float 1/S
        if constexpr (DO_Q) {
            // x_i = e_i fw / S: hand fuse_row the partition sum expressed in this wave's units
            const FuseRow fr = fuse_row(fw > 0.0 ? S / fw : 1.0, A.a, A.b);
            double q5[5];
            bool tiny = false;
            if constexpr (NVEC == 1) tiny = V <= kTinyVocab;       // uniform
            if (tiny) {
                if constexpr (NVEC == 1) {
                    if constexpr (RAD) {
                        __builtin_amdgcn_sched_barrier(0);
                        load_row(buf, A.radius, row);
                        E::zero_tail(buf[0], tid * EPV, V);
                    }
                    fuse_sums_tiny<T, EPV, RAD>(e, buf[0], fw > 0.0 ? S / fw : 1.0, A.a, A.b, A.kappa, A.rmax, q5);
#pragma unroll
                    for (int i = 0; i < 5; ++i) q5[i] = wave_sum(q5[i]);
                }
            } else if constexpr (RAD) {
                // the raw radius row comes into the registers the centre row came in
                __builtin_amdgcn_sched_barrier(0);
                load_row(buf, A.radius, row);
                if (partial) {
#pragma unroll
                    for (int j = 0; j < NVEC; ++j) E::zero_tail(buf[j], (j * THREADS + tid) * EPV, V);
                }
                fuse_sums_rad<T, THREADS, NVEC>(e, buf, fr, (float)A.kappa, (float)A.rmax, V, q5);
#pragma unroll
                for (int i = 0; i < 5; ++i) q5[i] = wave_sum(q5[i]);
            } else if (capless) {
                if (split) fuse_sums<THREADS, NVEC, EPV, true, true>(e, fr, V, q5);
                else       fuse_sums<THREADS, NVEC, EPV, true, false>(e, fr, V, q5);
                q5[1] = wave_sum(q5[1]);
                q5[3] = wave_sum(q5[3]);
            } else {
                fuse_sums<THREADS, NVEC, EPV, false, true>(e, fr, V, q5);
#pragma unroll
                for (int i = 0; i < 5; ++i) q5[i] = wave_sum(q5[i]);
            }
            if (lane == 0) {
                const double f2 = fw * fw;
                sm_q5[wave * 5 + 0] = q5[0] * fw; sm_q5[wave * 5 + 1] = q5[1] * fw;
                sm_q5[wave * 5 + 2] = q5[2] * f2; sm_q5[wave * 5 + 3] = q5[3] * f2; sm_q5[wave * 5 + 4] = q5[4] * f2;
            }
        }

        // ---- T: verifier row statistics, per wave; the row is not kept -------------------------------------
        if constexpr (DO_V) {
            float ntw;
            double Zw;
            // The verifier row is fetched only now, into the registers the centre row came in.  Fetching
            // it earlier, next to the interval pass, was measured slower: the other resident workgroups
            // already keep the memory system busy, and more loads in flight per wave only lengthen queues.
            __builtin_amdgcn_sched_barrier(0);
            load_row(buf, A.target, row);
            verifier_stats(buf, ntw, Zw);
            if (lane == 0) { sm_nt[wave] = ntw; sm_Z[wave] = Zw; }
        }
        // the next centre row goes in flight before the barrier and thread 0's bookkeeping
        __builtin_amdgcn_sched_barrier(0);
        if (has_next) load_row(buf, A.draft, next);

        // ---- thread 0 leaves the row's ten numbers for the finishing kernels -------------------------------
        __syncthreads();
        if (tid == 0) {
            float nt = -INFINITY;
            double Z = 0.0;                                        // in units of 2^-nt
            if constexpr (DO_V) {
#pragma unroll
                for (int w = 0; w < NW; ++w) nt = fmaxf(nt, sm_nt[w]);
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float rt = sm_nt[w];
                    if (rt != -INFINITY) Z += sm_Z[w] * pow2_of(rt - nt);
                }
            }
            RowStats* st = A.stats + row;
            st->S = S; st->Z = Z; st->n = n; st->nt = nt; st->mc = mc; st->capless = capless ? 1.f : 0.f;
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                double t = 0.0;
                if constexpr (DO_Q) {
#pragma unroll
                    for (int w = 0; w < NW; ++w) t += sm_q5[w * 5 + i];
                }
                st->q[i] = t;
            }
        }

        if (!has_next) break;
        row = next;
    }
}

// ---- the finishing kernels ----------------------------------------------------------------------------------------

// Window w = rows [wK, min((w+1)K, N)): accepted prefix length and the draw of the first rejected row
// (Algorithm 1: the verified part of a drafted window and the token that replaces the first rejection).
__device__ __forceinline__ void window_of(const uint8_t* accept, const int32_t* row_id, int64_t N, int32_t K,
                                          int64_t w, int32_t* accept_len, int32_t* resampled_id)
{
    const int64_t lo = w * K;
    const int64_t hi = (lo + K < N) ? lo + K : N;
    int64_t n = 0;
    while (lo + n < hi && accept[lo + n]) ++n;
    if (accept_len) accept_len[w] = (int32_t)n;
    if (resampled_id)
        resampled_id[w] = (lo + n < hi) ? row_id[lo + n] : -1;
}

// One thread per row: RowStats -> the row's outputs, in fp64 (Eq. uncertainty_score; Algorithm 1's threshold
// and verification steps).  Rejected rows are appended to a list for the residual draw.
// A workgroup covers `rows_per_block` consecutive rows.  When the window outputs are asked for, that is a
// multiple of the window length K, so every window lies inside one workgroup: its leader thread counts the
// accepted prefix from the accept bits the workgroup shares through LDS, and writes -1 for a window
// without a rejection (the draw of a window with one is written by the residual-draw kernel).
template <typename T>
__global__ __launch_bounds__(256) void rowfinish_kernel(const RowArgs A, const int do_q, const int do_v,
                                                        const int rows_per_block, const int K,
                                                        int32_t* __restrict__ accept_len,
                                                        int32_t* __restrict__ resampled_id)
{
    __shared__ uint8_t sm_acc[256];
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * rows_per_block + tid;
    const bool live = tid < rows_per_block && row < A.N;
    const bool windows = accept_len || resampled_id;               // uniform over the grid
    int rej = 0;
    if (live) {
        const int V = A.V;
        const T* crow = static_cast<const T*>(A.draft) + row * A.stride;
        const RowStats st = A.stats[row];
        const double S = st.S;
        const float n = st.n;

        int xid = -1;
        float cx = st.mc;                                          // no ids: the arg-max token is reported
        if (A.ids) {
            xid = A.ids[row];
            xid = xid < 0 ? 0 : (xid >= V ? V - 1 : xid);
            cx = load_logit(crow, xid);
        }
        if (do_q) {
            const RowScore rs = finish_score(st.q, S, st.capless != 0.f, A);
            if (A.omega) A.omega[row] = (float)rs.omega;
            if (A.sigma) A.sigma[row] = (float)rs.sigma;
            if (A.score) A.score[row] = (float)rs.score;
            if (A.flags) A.flags[row] = (uint8_t)(rs.score > A.tau);
            if (A.p_lo || A.p_mid || A.p_hi) {
                const double x = exp((double)cx - (double)n * kLn2) / S;
                double a = A.a, b = A.b;
                if (A.radius) {
                    // the reported token's own radius (the launcher supplies ids in this mode)
                    const T* rrow = static_cast<const T*>(A.radius) + row * A.stride;
                    const double r = radius_of((double)load_logit(rrow, xid < 0 ? 0 : xid), A.kappa, A.rmax);
                    a = exp(r); b = exp(-r);
                }
                if (A.p_mid) A.p_mid[row] = (float)x;
                if (A.p_lo) A.p_lo[row] = (float)(rs.alpha_l * b * x / (1.0 + (b - 1.0) * x));
                if (A.p_hi) A.p_hi[row] = (float)(rs.alpha_u * a * x / (1.0 + (a - 1.0) * x));
            }
        }
        if (do_v) {
            // ln p_x = cx - n ln2 - ln S, ln q_x = tx - nt ln2 - ln Z;  accept iff ln u < min(0, ln q_x - ln p_x)
            const T* trow = static_cast<const T*>(A.target) + row * A.stride;
            const float tx = load_logit(trow, xid);
            const double lp = ((double)cx - (double)n * kLn2) - log(S);
            const double lq = ((double)tx - (double)st.nt * kLn2) - log(st.Z);
            const double lnu = log((double)A.u_accept[row]);       // log(0) = -inf: always accepted
            rej = !(lnu < fmin(0.0, lq - lp));
            if (A.accept) A.accept[row] = (uint8_t)(!rej);
            if (A.row_id && !rej) A.row_id[row] = -1;
        }
    }
    bool first = false;                                            // first rejection of its window
    if (windows) {
        sm_acc[tid] = (uint8_t)(!rej);
        __syncthreads();
        const int lead = tid - tid % K;                            // block starts are multiples of K
        if (live && tid == lead) {
            const int64_t left = A.N - row;
            const int len = (int)(left < K ? left : K);
            int m = 0;
            while (m < len && sm_acc[tid + m]) ++m;
            const int64_t w = row / K;
            if (accept_len) accept_len[w] = m;
            if (resampled_id && m == len) resampled_id[w] = -1;
        }
        if (rej) {
            first = true;
            for (int i = lead; i < tid; ++i) first = first && sm_acc[i] != 0;
        }
    }
    if (rej && A.row_id) {
        // list entry: the row, bit-complemented when the row's draw is also its window's
        const int slot = atomicAdd(A.reject_count, 1);
        if (slot < A.N) A.reject_list[slot] = first ? ~(int32_t)row : (int32_t)row;   // (one entry per row at most)
    }
}

// Residual draw of the rejected rows: res_i = max(0, q_i - p_i), inverse CDF in token order.  Workgroups walk
// over the list of rejected rows; both rows are fetched again (they were read moments ago: mostly from
// cache), four vectors of each row per lane in flight at once.  A row's draw is a chain of dependent
// steps (list entry, statistics, loads, totals, crossing chunk, scan), so what matters is how many rows
// a compute unit has in flight: 256-lane workgroups, several per compute unit, unless the launch is so
// small that most compute units would see no rejected row at all (then 1024 lanes work on each row).
template <typename T, int THREADS>
__global__ __launch_bounds__(THREADS) void resample_kernel(const RowArgs A, const int K, int32_t* __restrict__ resampled_id)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec;
    constexpr int NW = THREADS / 64;
    constexpr int CHUNK = THREADS * EPV;
    constexpr int MAXCH = 8192 / THREADS;           // chunks of CHUNK tokens a row can have (supported vocabularies)
    constexpr int UB = 4;                           // chunks of each row in flight per lane

    __shared__ double sm_e[NW * MAXCH + NW];
    __shared__ int    sm_i[NW * 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = A.V;
    const int last_vec = (V + EPV - 1) / EPV - 1;
    const int nch = (V + CHUNK - 1) / CHUNK;        // <= MAXCH
    int count = *A.reject_count;
    if (count > A.N) count = (int)A.N;

    for (int item = blockIdx.x; item < count; item += gridDim.x) {
        const int32_t entry = A.reject_list[item];
        const int64_t row = entry < 0 ? ~entry : entry;
        const T* crow = static_cast<const T*>(A.draft) + row * A.stride;
        const T* trow = static_cast<const T*>(A.target) + row * A.stride;
        const RowStats st = A.stats[row];
        const double invS = 1.0 / st.S, invZ = 1.0 / st.Z;
        const float n = st.n, nt = st.nt;
        const double u_res = (double)A.u_resample[row];

        auto load_vec = [&](const T* base, int j) -> u32x4 {
            const uint32_t off = (uint32_t)min(j * THREADS + tid, last_vec) * 16u;
            return *(gvec)((gbytes)base + off);
        };
        // residuals of one 16-byte vector of each row; tokens past the end of the row are masked to -inf
        auto residuals = [&](u32x4 cr, u32x4 tr, int j, float (&r)[EPV]) {
            E::mask_tail(cr, (j * THREADS + tid) * EPV, V);
            E::mask_tail(tr, (j * THREADS + tid) * EPV, V);
            float cv[EPV], tv[EPV];
            E::unpack(cr, cv);
            E::unpack(tr, tv);
#pragma unroll
            for (int k = 0; k < EPV; ++k) {
                const double q = (double)exp2_ref(tv[k], nt) * invZ;
                const double p = (double)exp2_ref(cv[k], n) * invS;
                r[k] = (float)fmax(q - p, 0.0);
            }
        };
        // E1: workgroup totals of the residual over each chunk of CHUNK tokens, UB chunks of each row in flight
        for (int j0 = 0; j0 < nch; j0 += UB) {
            u32x4 cb[UB], tb[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) { cb[u] = load_vec(crow, j0 + u); tb[u] = load_vec(trow, j0 + u); }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                if (j0 + u < nch) {                                // uniform
                    float r[EPV];
                    residuals(cb[u], tb[u], j0 + u, r);
                    float s = 0.f;
#pragma unroll
                    for (int k = 0; k < EPV; ++k) s += r[k];
                    const double ws = wave_sum((double)s);
                    if (lane == 0) sm_e[wave * MAXCH + j0 + u] = ws;
                }
            }
        }
        __syncthreads();
        double R = 0.0;
        for (int j = 0; j < nch; ++j) {
#pragma unroll
            for (int w = 0; w < NW; ++w) R += sm_e[w * MAXCH + j];
        }
        int cand = INT_MAX, lastpos = -1;
        if (R > 0.0) {
            // chunk that holds the crossing of u * R (token order = chunk order, then lane order)
            const double thr = u_res * R;
            int jstar = -1, jlast = 0;
            double before = 0.0, run = 0.0;
            for (int j = 0; j < nch; ++j) {
                double tot = 0.0;
#pragma unroll
                for (int w = 0; w < NW; ++w) tot += sm_e[w * MAXCH + j];
                if (jstar < 0 && run + tot > thr) { jstar = j; before = run; }
                if (tot > 0.0) jlast = j;
                if (jstar < 0) run += tot;
            }
            if (jstar < 0) { jstar = jlast; before = run; }        // unreachable for u < 1; keeps the draw valid
            // E2: the lane's residuals inside that chunk, fetched again (cache) and recomputed exactly as in E1
            float r[EPV];
            residuals(load_vec(crow, jstar), load_vec(trow, jstar), jstar, r);
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < EPV; ++k) s += r[k];
            const double incl = wave_scan((double)s);
            if (lane == 63) sm_e[NW * MAXCH + wave] = incl;
            __syncthreads();
            double cum = before + (incl - (double)s);
            for (int w = 0; w < wave; ++w) cum += sm_e[NW * MAXCH + w];
            // smallest token of the chunk whose inclusive running sum exceeds u * R; tokens without
            // residual mass cannot be drawn; lastpos covers a crossing lost to rounding at the chunk end
            const int base = (jstar * THREADS + tid) * EPV;
#pragma unroll
            for (int k = 0; k < EPV; ++k) {
                cum += (double)r[k];
                if (r[k] > 0.f) {
                    lastpos = base + k;
                    if (cum > thr && cand == INT_MAX) cand = base + k;
                }
            }
        } else {
            // every residual rounded to zero (q == p to working precision): the draw degenerates to the
            // lowest-index arg-max of q; this path is practically never taken
            float mt = -INFINITY;
            for (int i = tid; i < V; i += THREADS) mt = fmaxf(mt, load_logit(trow, i));
            mt = wave_max(mt);
            if (lane == 0) sm_e[NW * MAXCH + wave] = (double)mt;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < NW; ++w) mt = fmaxf(mt, (float)sm_e[NW * MAXCH + w]);
            for (int i = tid; i < V; i += THREADS)
                if (load_logit(trow, i) == mt) { cand = i; break; }
        }
        cand = wave_min_i(cand);
        lastpos = wave_max_i(lastpos);
        if (lane == 0) { sm_i[wave * 2] = cand; sm_i[wave * 2 + 1] = lastpos; }
        __syncthreads();
        if (tid == 0) {
            int c0 = sm_i[0], l0 = sm_i[1];
#pragma unroll
            for (int w = 1; w < NW; ++w) { c0 = min(c0, sm_i[w * 2]); l0 = max(l0, sm_i[w * 2 + 1]); }
            int id = (c0 != INT_MAX) ? c0 : l0;
            if (id < 0) id = 0;
            A.row_id[row] = id;
            if (entry < 0 && resampled_id) resampled_id[row / K] = id;             // the window's draw is its first rejected row's
        }
        __syncthreads();                                           // the LDS slots are reused by the next row
    }
}

// ---- arg-max token of every row (tensor-radius calls without drafted ids) ----------------------------------

// One workgroup per row: the lowest index that holds the row's largest centre logit.  Only the
// tensor-radius mode needs the index itself (to pick that token's radius); the scalar mode reports the
// arg-max token from the row maximum alone.
template <typename T>
__global__ __launch_bounds__(256) void argmax_kernel(const RowArgs A, int32_t* __restrict__ out)
{
    __shared__ float sm_m[4];
    __shared__ int sm_i[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const T* c = static_cast<const T*>(A.draft) + row * A.stride;
    float m = -INFINITY;
    int idx = INT_MAX;
    for (int i = tid; i < A.V; i += 256) {
        const float v = load_logit(c, i);
        if (v > m || idx == INT_MAX) { m = v; idx = i; }           // ascending i: the first of equal values stays
    }
    const float wm = wave_max(m);
    const int wi = wave_min_i(m == wm ? idx : INT_MAX);
    if (lane == 0) { sm_m[wave] = wm; sm_i[wave] = wi; }
    __syncthreads();
    if (tid == 0) {
        const float rm = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));
        int best = INT_MAX;
        for (int w = 0; w < 4; ++w) if (sm_m[w] == rm && sm_i[w] < best) best = sm_i[w];
        out[row] = best == INT_MAX ? 0 : best;
    }
}

// ---- several heads (Sec. 4, ablation on the Inter-Head): Ensemble and Voting ------------------------------

constexpr int kMaxHeads = 8;

// Ensemble: the heads' curves are averaged token by token, so the widths of all heads of a token have to
// meet: a second sweep over the H rows of a position, after the streaming kernel has left every head's
// RowStats (partition sum, reference, interval sums -> that head's caps).  One workgroup per position;
// per token and head the same arithmetic as the streaming kernel's interval pass.
//   D_i = sum_h delta_{h,i},  Omega = sum_i D_i / H,  Sigma^2 = sum_i D_i^2 / (H^2 V) - (Omega / V)^2.
template <typename T>
__global__ __launch_bounds__(256) void ensemble_kernel(const RowArgs A, const int H, const int64_t head_stride)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec;
    __shared__ FuseRow sm_fr[kMaxHeads];
    __shared__ float sm_n[kMaxHeads], sm_invS[kMaxHeads];
    __shared__ double sm_cw[kMaxHeads], sm_cl[kMaxHeads], sm_S[kMaxHeads], sm_al[kMaxHeads], sm_au[kMaxHeads];
    __shared__ double sm_red[2][4];
    __shared__ float sm_pm[4];
    __shared__ int sm_pi[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = A.V;
    const bool rad = A.radius != nullptr;
    const bool need_argmax = A.ids == nullptr && (A.p_lo || A.p_mid || A.p_hi);
    const bool tiny = V <= 64;

    if (tid < H) {
        const RowStats st = A.stats[(int64_t)tid * A.N + row];
        const RowScore rs = finish_score(st.q, st.S, st.capless != 0.f, A);
        const double Bc = (rad ? 1.0 : A.b) / st.S, Wc = (rad ? 1.0 : A.a - A.b) / st.S;
        sm_fr[tid] = fuse_row(st.S, A.a, A.b);
        sm_n[tid] = st.n;
        sm_cw[tid] = rs.alpha_u * Wc;
        sm_cl[tid] = (rs.alpha_u - rs.alpha_l) * Bc;
        sm_invS[tid] = (float)(1.0 / st.S);
        sm_S[tid] = st.S; sm_al[tid] = rs.alpha_l; sm_au[tid] = rs.alpha_u;
    }
    __syncthreads();

    const float kap = (float)A.kappa, rmax = (float)A.rmax;
    const int nvec = (V + EPV - 1) / EPV;
    double s1 = 0.0, s2 = 0.0;
    float best = -INFINITY;
    int best_i = INT_MAX;
    if (tiny) {
        // A handful of tokens (one vector per lane at most): widths are O(1) and Sigma can be an exact zero
        // (two tokens), which fp32 token arithmetic cannot resolve to 1e-7; the few tokens are done in fp64.
        if (tid < nvec) {
            double D[EPV];
            float pm[EPV];
#pragma unroll
            for (int k = 0; k < EPV; ++k) { D[k] = 0.0; pm[k] = 0.f; }
            for (int h = 0; h < H; ++h) {
                const gvec c = (gvec)(gbytes)(static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride);
                const gvec r = (gvec)(gbytes)(static_cast<const T*>(rad ? A.radius : A.draft) +
                                              (int64_t)h * head_stride + row * A.stride);
                const u32x4 cw4 = c[tid], rw4 = r[tid];
                float cv[EPV], rv[EPV];
                E::unpack(cw4, cv);
                E::unpack(rw4, rv);
                for (int k = 0; k < EPV; ++k) {
                    if (tid * EPV + k < V) {
                        const double x = exp((double)cv[k] - (double)sm_n[h] * kLn2) / sm_S[h];
                        double a = A.a, b = A.b;
                        if (rad) {
                            const double rr = radius_of((double)rv[k], A.kappa, A.rmax);
                            a = exp(rr); b = exp(-rr);
                        }
                        D[k] += sm_au[h] * a * x / (1.0 + (a - 1.0) * x) - sm_al[h] * b * x / (1.0 + (b - 1.0) * x);
                        pm[k] += (float)x;
                    }
                }
            }
            for (int k = 0; k < EPV; ++k) {
                const int tok = tid * EPV + k;
                s1 += D[k];
                s2 = fma(D[k], D[k], s2);
                if (need_argmax && tok < V && pm[k] > best) { best = pm[k]; best_i = tok; }
            }
        }
    }
    constexpr int UB = 16 / EPV;                                   // vectors of a head in flight per lane
    for (int v0 = tid; !tiny && v0 < nvec; v0 += 256 * UB) {
        double D[UB][EPV];                                         // fp64 across heads
        float pm[UB][EPV];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
#pragma unroll
            for (int k = 0; k < EPV; ++k) { D[u][k] = 0.0; pm[u][k] = 0.f; }
        }
        for (int h = 0; h < H; ++h) {
            const gvec c = (gvec)(gbytes)(static_cast<const T*>(A.draft) + (int64_t)h * head_stride + row * A.stride);
            const gvec r = (gvec)(gbytes)(static_cast<const T*>(rad ? A.radius : A.draft) + (int64_t)h * head_stride +
                                          row * A.stride);
            u32x4 cw4[UB], rw4[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) cw4[u] = c[min(v0 + u * 256, nvec - 1)];
            if (rad) {
#pragma unroll
                for (int u = 0; u < UB; ++u) rw4[u] = r[min(v0 + u * 256, nvec - 1)];
            }
            const FuseRow fr = sm_fr[h];
            const float n = sm_n[h], invS = sm_invS[h];
            const double cw = sm_cw[h], cl = sm_cl[h];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int tok0 = (v0 + u * 256) * EPV;             // >= V for vectors past the row's end
                float cv[EPV], rv[EPV];
                E::unpack(cw4[u], cv);
                if (rad) E::unpack(rw4[u], rv);
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    if (tok0 + k < V) {
                        const float e = exp2_ref(cv[k], n);
                        float gl, gw;
                        if (rad) fuse_token_rad(e, rv[k], fr, kap, rmax, gl, gw);
                        else fuse_token(e, fr, gl, gw);
                        D[u][k] = fma(cw, (double)gw, fma(cl, (double)gl, D[u][k]));
                        pm[u][k] = fmaf(e, invS, pm[u][k]);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
#pragma unroll
            for (int k = 0; k < EPV; ++k) {
                const int tok = (v0 + u * 256) * EPV + k;
                const double d = D[u][k];                          // tokens past V contribute exactly 0
                s1 += d;
                s2 = fma(d, d, s2);
                if (need_argmax && tok < V && pm[u][k] > best) { best = pm[u][k]; best_i = tok; }
            }
        }
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (lane == 0) { sm_red[0][wave] = s1; sm_red[1][wave] = s2; }
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
        const double omega = t1 / Hd;
        const double var = fmax(0.0, t2 / (Hd * Hd) - omega * omega / Vd) / Vd;
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
                const double x = exp((double)load_logit(crow, xid) - (double)sm_n[h] * kLn2) / sm_S[h];
                double a = A.a, b = A.b;
                if (rad) {
                    const T* rrow = static_cast<const T*>(A.radius) + (int64_t)h * head_stride + row * A.stride;
                    const double r = radius_of((double)load_logit(rrow, xid), A.kappa, A.rmax);
                    a = exp(r); b = exp(-r);
                }
                mid += x;
                lo += sm_al[h] * b * x / (1.0 + (b - 1.0) * x);
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

// ---- Inter-DRO loss, forward (Sec. 3.2.3: anchor, DRO and alignment equations) -----------------------------

// r = min(kappa Softplus(raw), rmax) in fp32 (see radius_ab for the ln(1 + t) form).
__device__ __forceinline__ float radius_r(float raw, float kappa, float rmax)
{
    const float t = __builtin_amdgcn_exp2f(-fabsf(raw) * 1.44269504f);
    const float u = 1.0f + t;
    const float d = u - 1.0f;
    const float lg = d == 0.f ? t : (__builtin_amdgcn_logf(u) * 0.693147181f) * (t * __builtin_amdgcn_rcpf(d));
    return fminf(kappa * (fmaxf(raw, 0.f) + lg), rmax);
}

// Per-row terms of the loss.  One 1024-lane workgroup per row holds the centre, raw-radius and cloud rows as
// loaded (12 registers per vector) and makes three passes over them: the four maxima (of c, c + r, c - r and
// the cloud logits), the four partition sums together with sum p_cloud o for the cross-entropies, and the
// three L1 distances, which need all four normalisers.  With e = 2^(o log2e - n), n = ceil(max log2e):
//   CE(p_cloud, softmax(o)) = (n ln2 + ln S_o) - (sum_i et_i o_i) / Z,
//   KL(p_cloud || p_mid)    = (sum_i et_i t_i) / Z - (nt ln2 + ln Z) + CE(p_cloud, p_mid).
// terms[k * N + row], k = 0..6: L1(mid), L1(up), L1(lo), CE(mid), CE(up), CE(lo), KL.
template <typename T, int NVEC>
__global__ __launch_bounds__(1024) void dro_row_kernel(const RowArgs A, float* __restrict__ terms)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec, THREADS = 1024, NW = 16;
    __shared__ float sm_f[NW * 4];
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
        cw[j] = *(gvec)(cb + off);
        tw[j] = *(gvec)(tb + off);
        if (rad) rw[j] = *(gvec)(rb + off);
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
    auto block_max4 = [&](float (&m)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) m[i] = wave_max(m[i]);
        if (lane == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) sm_f[wave * 4 + i] = m[i];
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = sm_f[i];
#pragma unroll 1
            for (int w = 1; w < NW; ++w) v = fmaxf(v, sm_f[w * 4 + i]);
            m[i] = v;
        }
    };

    // pass 1: maxima -> integer references
    float mx[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float c, r, t;
            element(j, k, c, r, t);
            mx[0] = fmaxf(mx[0], c); mx[1] = fmaxf(mx[1], c + r); mx[2] = fmaxf(mx[2], c - r); mx[3] = fmaxf(mx[3], t);
        }
    }
    block_max4(mx);
    float nref[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { nref[i] = ref_of(mx[i]); if (nref[i] == -INFINITY) nref[i] = 0.f; }

    // pass 2: partition sums and the p_cloud-weighted sums of c, r and the cloud logits
    fresh();
    double acc[7] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};          // S_mid, S_up, S_lo, Z, sum et c, sum et r, sum et t
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float c, r, t;
            element(j, k, c, r, t);
            const float et = exp2_ref(t, nref[3]);
            acc[0] += (double)exp2_ref(c, nref[0]);
            acc[1] += (double)exp2_ref(c + r, nref[1]);
            acc[2] += (double)exp2_ref(c - r, nref[2]);
            acc[3] += (double)et;
            if (et > 0.f) {                                        // a token the cloud rules out weighs nothing
                acc[4] = fma((double)et, (double)c, acc[4]);
                acc[5] = fma((double)et, (double)r, acc[5]);
                acc[6] = fma((double)et, (double)t, acc[6]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < 7; ++i) acc[i] = wave_sum(acc[i]);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < 7; ++i) sm_d[wave * 7 + i] = acc[i];
    }
    __syncthreads();
    double tot[7];
#pragma unroll
    for (int i = 0; i < 7; ++i) {
        double v = 0.0;
#pragma unroll 1
        for (int w = 0; w < NW; ++w) v += sm_d[w * 7 + i];
        tot[i] = v;
    }
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
            const float pc = exp2_ref(t, nref[3]) * iz;
            l1[0] += (double)fabsf(exp2_ref(c, nref[0]) * is0 - pc);
            l1[1] += (double)fabsf(exp2_ref(c + r, nref[1]) * is1 - pc);
            l1[2] += (double)fabsf(exp2_ref(c - r, nref[2]) * is2 - pc);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < 3; ++i) l1[i] = wave_sum(l1[i]);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < 3; ++i) sm_d[wave * 7 + i] = l1[i];
    }
    __syncthreads();
    if (tid == 0) {
        double L[3] = {0.0, 0.0, 0.0};
#pragma unroll 1
        for (int w = 0; w < NW; ++w) { L[0] += sm_d[w * 7]; L[1] += sm_d[w * 7 + 1]; L[2] += sm_d[w * 7 + 2]; }
        const double Z = tot[3];
        const double pc_c = tot[4] / Z, pc_r = tot[5] / Z, pc_t = tot[6] / Z;
        const double ce_mid = ((double)nref[0] * kLn2 + log(tot[0])) - pc_c;
        const double ce_up = ((double)nref[1] * kLn2 + log(tot[1])) - (pc_c + pc_r);
        const double ce_lo = ((double)nref[2] * kLn2 + log(tot[2])) - (pc_c - pc_r);
        const double kl = pc_t - ((double)nref[3] * kLn2 + log(Z)) + ce_mid;
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

// ---- window epilogue: one thread per window of K rows -------------------------------------------------

__global__ __launch_bounds__(256) void window_kernel(const uint8_t* __restrict__ accept,
                                                     const int32_t* __restrict__ row_id, int64_t N, int32_t K,
                                                     int32_t* __restrict__ accept_len,
                                                     int32_t* __restrict__ resampled_id)
{
    const int64_t W = (N + K - 1) / K;
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= W) return;
    window_of(accept, row_id, N, K, w, accept_len, resampled_id);
}

// ---- dense export (tests / debugging): same per-token arithmetic, sweeps over global memory ---------------

template <typename T>
__global__ __launch_bounds__(256) void dense_kernel(const RowArgs A, float* __restrict__ p_lo,
                                                    float* __restrict__ p_mid, float* __restrict__ p_hi)
{
    constexpr int NW = 4;
    __shared__ double smem[NW];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = A.V;
    const T* c = static_cast<const T*>(A.draft) + row * A.stride;

    auto block_sum = [&](double v) -> double {
        v = wave_sum(v);
        __syncthreads();
        if (lane == 0) smem[wave] = v;
        __syncthreads();
        return (smem[0] + smem[1]) + (smem[2] + smem[3]);
    };

    float m = -INFINITY;
    for (int i = tid; i < V; i += 256) m = fmaxf(m, load_logit(c, i));
    m = wave_max(m);
    __syncthreads();
    if (lane == 0) smem[wave] = (double)m;
    __syncthreads();
    m = fmaxf(fmaxf((float)smem[0], (float)smem[1]), fmaxf((float)smem[2], (float)smem[3]));
    const float n = ref_of(m);

    double acc = 0.0;
    for (int i = tid; i < V; i += 256) acc += (double)exp2_ref(load_logit(c, i), n);
    const double S = block_sum(acc);

    const FuseRow fr = fuse_row(S, A.a, A.b);
    const T* rad = A.radius ? static_cast<const T*>(A.radius) + row * A.stride : nullptr;
    const float kap = (float)A.kappa, rmax = (float)A.rmax;
    // gl, gw of one token: p^l = Bc gl, p^u - p^l = Wc gw (tensor-radius mode: Bc = Wc = 1 / S)
    auto token = [&](int i, float& e, float& gl, float& gw) {
        e = exp2_ref(load_logit(c, i), n);
        if (rad) fuse_token_rad(e, load_logit(rad, i), fr, kap, rmax, gl, gw);
        else fuse_token(e, fr, gl, gw);
    };
    double q5[5];
    {
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0, a4 = 0.0;
        for (int i = tid; i < V; i += 256) {
            float e, gl, gw;
            token(i, e, gl, gw);
            const double dl = (double)gl, dw = (double)gw;
            a0 += dl; a1 += dw;
            a2 = fma(dl, dl, a2); a3 = fma(dw, dw, a3); a4 = fma(dl, dw, a4);
        }
        q5[0] = block_sum(a0); q5[1] = block_sum(a1); q5[2] = block_sum(a2);
        q5[3] = block_sum(a3); q5[4] = block_sum(a4);
    }
    const RowScore rs = finish_score(q5, S, false, A);

    const float Bc = (float)((rad ? 1.0 : A.b) / S), Wc = (float)((rad ? 1.0 : A.a - A.b) / S), invS = (float)(1.0 / S);
    const float al = (float)rs.alpha_l, au = (float)rs.alpha_u;
    for (int i = tid; i < V; i += 256) {
        float e, gl, gw;
        token(i, e, gl, gw);
        const float pl = Bc * gl;
        const float pu = fmaf(Wc, gw, pl);
        const int64_t o = row * (int64_t)V + i;
        if (p_lo) p_lo[o] = al * pl;
        if (p_mid) p_mid[o] = e * invS;
        if (p_hi) p_hi[o] = au * pu;
    }
}

// ---- plain streaming read: the bandwidth ceiling the streaming kernel is held against ---------------------

// One workgroup per row: every 16-byte vector of the row pair is loaded once, with up to 2 x 8 loads per
// lane in flight, and summed as floats.  No exponentials, no exchange beyond one reduction per row.
template <typename T>
__global__ __launch_bounds__(256) void read_kernel(const RowArgs A, float* __restrict__ row_sum)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec, UB = 8;
    __shared__ float sm[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = A.V;
    const int nvec = (V + EPV - 1) / EPV;
    const gvec c = (gvec)(gbytes)(static_cast<const T*>(A.draft) + row * A.stride);
    const gvec t = (gvec)(gbytes)(static_cast<const T*>(A.target ? A.target : A.draft) + row * A.stride);
    const bool two = A.target != nullptr;                          // uniform
    // Vectors past the end of the row are clamped to its last one and zeroed as loaded; so is the
    // padding inside the row's last vector.  Branch-free: a word survives iff its token exists.
    auto clean = [&](u32x4& r, int v) {
        const int first = v * EPV;
        if constexpr (EPV == 4) {
            r.x = first + 0 < V ? r.x : 0u;
            r.y = first + 1 < V ? r.y : 0u;
            r.z = first + 2 < V ? r.z : 0u;
            r.w = first + 3 < V ? r.w : 0u;
        } else {
            r.x &= (first + 0 < V ? 0x0000ffffu : 0u) | (first + 1 < V ? 0xffff0000u : 0u);
            r.y &= (first + 2 < V ? 0x0000ffffu : 0u) | (first + 3 < V ? 0xffff0000u : 0u);
            r.z &= (first + 4 < V ? 0x0000ffffu : 0u) | (first + 5 < V ? 0xffff0000u : 0u);
            r.w &= (first + 6 < V ? 0x0000ffffu : 0u) | (first + 7 < V ? 0xffff0000u : 0u);
        }
    };
    float acc0 = 0.f, acc1 = 0.f;
#pragma unroll 1
    for (int base = 0; base < nvec; base += UB * 256) {
        u32x4 cb[UB], tb[UB];
#pragma unroll
        for (int j = 0; j < UB; ++j) cb[j] = c[min(base + j * 256 + tid, nvec - 1)];
        if (two) {
#pragma unroll
            for (int j = 0; j < UB; ++j) tb[j] = t[min(base + j * 256 + tid, nvec - 1)];
        }
        const bool ragged = base + UB * 256 >= nvec;               // uniform: this sweep reaches the row's end
#pragma unroll
        for (int j = 0; j < UB; ++j) {
            if (ragged) {
                clean(cb[j], base + j * 256 + tid);
                if (two) clean(tb[j], base + j * 256 + tid);
            }
            float cv[EPV], tv[EPV];
            E::unpack(cb[j], cv);
#pragma unroll
            for (int k = 0; k < EPV; k += 2) { acc0 += cv[k]; acc1 += cv[k + 1]; }
            if (two) {
                E::unpack(tb[j], tv);
#pragma unroll
                for (int k = 0; k < EPV; k += 2) { acc0 += tv[k]; acc1 += tv[k + 1]; }
            }
            __builtin_amdgcn_sched_barrier(0);                     // unpack one vector at a time
        }
    }
    float acc = acc0 + acc1;
    acc = (float)wave_sum((double)acc);
    if (lane == 0) sm[wave] = acc;
    __syncthreads();
    if (tid == 0) row_sum[row] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

// ---- dispatch ---------------------------------------------------------------------------------------------

}  // namespace
hipError_t launch_windows(const uint8_t* accept, const int32_t* row_id, int64_t N, int32_t K,
                          int32_t* accept_len, int32_t* resampled_id, hipStream_t stream);
namespace {

// Compute units of the current device (asked once per device, then cached).
int compute_units()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    static int cache[64] = {0};
    if (cache[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        cache[dev] = cus;
    }
    return cache[dev];
}

template <typename T, int THREADS, int NVEC, bool DO_Q, bool DO_V, bool RAD>
hipError_t launch_stream_kernel(const RowArgs& a, hipStream_t s)
{
    // One wave of resident workgroups, each walking over rows with stride gridDim.x.  The register
    // budget the kernel was compiled for fixes how many fit: target_waves() waves per SIMD, and a
    // workgroup puts THREADS / 256 waves on each of the four SIMDs of a compute unit.
    constexpr int per_cu = target_waves<T, THREADS, NVEC, RAD>() / (THREADS / 256);
    const int64_t resident = (int64_t)per_cu * compute_units();
    const unsigned grid = (unsigned)(a.N < resident ? a.N : resident);
    hipLaunchKernelGGL((stream_kernel<T, THREADS, NVEC, DO_Q, DO_V, RAD>), dim3(grid), dim3(THREADS), 0, s, a);
    return hipGetLastError();
}

template <typename T, int THREADS, int NVEC>
hipError_t launch_stream_cfg(Mode mode, const RowArgs& a, hipStream_t s)
{
    const bool rad = a.radius != nullptr;
    switch (mode) {
    case Mode::Quantify: return rad ? launch_stream_kernel<T, THREADS, NVEC, true, false, true>(a, s)
                                    : launch_stream_kernel<T, THREADS, NVEC, true, false, false>(a, s);
    case Mode::Verify:   return launch_stream_kernel<T, THREADS, NVEC, false, true, false>(a, s);
    case Mode::Fused:    return rad ? launch_stream_kernel<T, THREADS, NVEC, true, true, true>(a, s)
                                    : launch_stream_kernel<T, THREADS, NVEC, true, true, false>(a, s);
    }
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_stream_typed(Mode mode, const RowArgs& a, hipStream_t s)
{
    const int vecs = (a.V + Elt<T>::kPerVec - 1) / Elt<T>::kPerVec;   // 16-byte vectors per row
    if (vecs <= 256 * 1)  return launch_stream_cfg<T, 256, 1>(mode, a, s);
    if (vecs <= 256 * 2)  return launch_stream_cfg<T, 256, 2>(mode, a, s);
    if (vecs <= 256 * 4)  return launch_stream_cfg<T, 256, 4>(mode, a, s);
    if (vecs <= 256 * 8)  return launch_stream_cfg<T, 256, 8>(mode, a, s);
    if (vecs <= 256 * 16) {
        // Few rows per workgroup: eight waves on a row keep the last rows of the launch short and the
        // grid even; with many rows the four-wave tile has less exchange overhead (measured).
        if (a.N < 12 * (int64_t)compute_units()) return launch_stream_cfg<T, 512, 8>(mode, a, s);
        return launch_stream_cfg<T, 256, 16>(mode, a, s);
    }
    if (vecs <= 1024 * 8) return launch_stream_cfg<T, 1024, 8>(mode, a, s);
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_finish_typed(Mode mode, const RowArgs& a, int32_t K, int32_t* accept_len, int32_t* resampled_id,
                               hipStream_t s)
{
    // Windows of up to 256 rows are finished inside the two kernels; longer ones by the window kernel.
    const bool want_windows = mode != Mode::Quantify && (accept_len || resampled_id);
    const bool inline_windows = want_windows && K <= 256 && (a.row_id || !resampled_id);
    const int rows_per_block = inline_windows ? (256 / K) * K : 256;
    const unsigned blocks = (unsigned)((a.N + rows_per_block - 1) / rows_per_block);
    hipLaunchKernelGGL(rowfinish_kernel<T>, dim3(blocks), dim3(256), 0, s, a, mode != Mode::Verify ? 1 : 0,
                       mode != Mode::Quantify ? 1 : 0, rows_per_block, K, inline_windows ? accept_len : nullptr,
                       inline_windows ? resampled_id : nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || mode == Mode::Quantify) return e;
    if (a.row_id) {
        const int64_t cus = compute_units();
        if (a.N >= 4 * cus) {
            // four 256-lane workgroups per compute unit walk over the rejected rows
            hipLaunchKernelGGL((resample_kernel<T, 256>), dim3((unsigned)(4 * cus)), dim3(256), 0, s, a, K,
                               inline_windows ? resampled_id : nullptr);
        } else {
            // very few rows (less than one rejected row per compute unit): 1024 lanes on each row
            const unsigned grid = (unsigned)(a.N < cus ? a.N : cus);
            hipLaunchKernelGGL((resample_kernel<T, 1024>), dim3(grid), dim3(1024), 0, s, a, K,
                               inline_windows ? resampled_id : nullptr);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (want_windows && !inline_windows)
        return launch_windows(a.accept, a.row_id, a.N, K, accept_len, resampled_id, s);
    return hipSuccess;
}

}  // namespace

int max_vocab(int dtype) { return dtype == 0 ? 1024 * 8 * 4 : 1024 * 8 * 8; }

hipError_t launch_stream(Mode mode, int dtype, const RowArgs& args, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    return dtype == 0 ? launch_stream_typed<float>(mode, args, stream)
                      : launch_stream_typed<bf16_t>(mode, args, stream);
}

hipError_t launch_finish(Mode mode, int dtype, const RowArgs& args, int32_t K, int32_t* accept_len,
                         int32_t* resampled_id, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    return dtype == 0 ? launch_finish_typed<float>(mode, args, K, accept_len, resampled_id, stream)
                      : launch_finish_typed<bf16_t>(mode, args, K, accept_len, resampled_id, stream);
}

hipError_t launch_windows(const uint8_t* accept, const int32_t* row_id, int64_t N, int32_t K,
                          int32_t* accept_len, int32_t* resampled_id, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    const int64_t W = (N + K - 1) / K;
    const unsigned blocks = (unsigned)((W + 255) / 256);
    hipLaunchKernelGGL(window_kernel, dim3(blocks), dim3(256), 0, stream, accept, row_id, N, K, accept_len,
                       resampled_id);
    return hipGetLastError();
}

hipError_t launch_dense(int dtype, const RowArgs& args, float* p_lo, float* p_mid, float* p_hi,
                        hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)args.N), block(256);
    if (dtype == 0) hipLaunchKernelGGL(dense_kernel<float>, grid, block, 0, stream, args, p_lo, p_mid, p_hi);
    else hipLaunchKernelGGL(dense_kernel<bf16_t>, grid, block, 0, stream, args, p_lo, p_mid, p_hi);
    return hipGetLastError();
}

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

int max_heads() { return kMaxHeads; }

hipError_t launch_ensemble(int dtype, const RowArgs& args, int heads, int64_t head_stride, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)args.N), block(256);
    if (dtype == 0) hipLaunchKernelGGL(ensemble_kernel<float>, grid, block, 0, stream, args, heads, head_stride);
    else hipLaunchKernelGGL(ensemble_kernel<bf16_t>, grid, block, 0, stream, args, heads, head_stride);
    return hipGetLastError();
}

hipError_t launch_vote(const uint8_t* head_flags, int heads, int64_t N, uint8_t* flags, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(vote_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, stream, head_flags, heads, N, flags);
    return hipGetLastError();
}

hipError_t launch_argmax(int dtype, const RowArgs& args, int32_t* out, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)args.N), block(256);
    if (dtype == 0) hipLaunchKernelGGL(argmax_kernel<float>, grid, block, 0, stream, args, out);
    else hipLaunchKernelGGL(argmax_kernel<bf16_t>, grid, block, 0, stream, args, out);
    return hipGetLastError();
}

hipError_t launch_read(int dtype, const RowArgs& args, float* row_sum, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)args.N), block(256);
    if (dtype == 0) hipLaunchKernelGGL(read_kernel<float>, grid, block, 0, stream, args, row_sum);
    else hipLaunchKernelGGL(read_kernel<bf16_t>, grid, block, 0, stream, args, row_sum);
    return hipGetLastError();
}

}  // namespace ciar
