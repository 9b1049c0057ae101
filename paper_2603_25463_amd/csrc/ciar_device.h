// Device-side helpers shared by the gfx950 kernels of the library: element types, exact-by-construction
// exponentials, wave reductions, the per-token InterFuse arithmetic and the per-row finishing formulas.
// Internal; included by the .hip files only.
#pragma once

#include "ciar_internal.h"

#include <limits.h>
#include <atomic>
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

// Element offset of row r from the start of a logit tensor, and the index of its drafted token (see RowArgs:
// several heads in one launch).  Rows are counted in 32 bits (the entry points reject more).
__device__ __forceinline__ int64_t row_offset(const RowArgs& A, int64_t r)
{
    if (A.head_rows == 0) return r * A.stride;
    const uint32_t h = (uint32_t)r / (uint32_t)A.head_rows;
    return (int64_t)h * A.head_stride + (int64_t)((uint32_t)r - h * (uint32_t)A.head_rows) * A.stride;
}
__device__ __forceinline__ int64_t ids_index(const RowArgs& A, int64_t r)
{
    return A.ids_period ? (int64_t)((uint32_t)r % (uint32_t)A.ids_period) : r;
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

// Three sums over the wave at once, handed to every lane, in two steps so that the values need not be there at the same
// time.  wave_sum3_put: two DPP steps leave every quad's sum in its lanes and the quad leaders put it into row `which`
// of the wave's 48 slots of LDS.  wave_sum3_get: lane l < 48 takes slot l and one reduction over each row of 16 lanes
// finishes all three (a wave's LDS operations complete in order: no barrier).  ~45 instructions where three
// reductions of one double each are ~110, and nothing is held in registers between the two steps.
__device__ __forceinline__ void wave_sum3_put(double v, double* slots, int which, int lane)
{
    v = dpp_add<0xB1, 0xf>(v);                     // lane ^ 1  (quad_perm 1,0,3,2)
    v = dpp_add<0x4E, 0xf>(v);                     // lane ^ 2  (quad_perm 2,3,0,1)
    if ((lane & 3) == 0) slots[16 * which + (lane >> 2)] = v;
}
__device__ __forceinline__ void wave_sum3_get(const double* slots, int lane, double& a, double& b, double& c)
{
    double x = slots[lane < 48 ? lane : 0];
    x = lane < 48 ? x : 0.0;
    x = dpp_add<kRowShr1, 0xf>(x);
    x = dpp_add<kRowShr2, 0xf>(x);
    x = dpp_add<kRowShr4, 0xf>(x);
    x = dpp_add<kRowShr8, 0xf>(x);
    const int lo = __double2loint(x), hi = __double2hiint(x);
    a = __hiloint2double(__builtin_amdgcn_readlane(hi, 15), __builtin_amdgcn_readlane(lo, 15));
    b = __hiloint2double(__builtin_amdgcn_readlane(hi, 31), __builtin_amdgcn_readlane(lo, 31));
    c = __hiloint2double(__builtin_amdgcn_readlane(hi, 47), __builtin_amdgcn_readlane(lo, 47));
}

// sum over lanes 0..15 (the first DPP row), handed to every lane of the wave
__device__ __forceinline__ double row16_sum(double v)
{
    v = dpp_add<kRowShr1, 0xf>(v);
    v = dpp_add<kRowShr2, 0xf>(v);
    v = dpp_add<kRowShr4, 0xf>(v);
    v = dpp_add<kRowShr8, 0xf>(v);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 15);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 15);
    return __hiloint2double(hi, lo);
}

// the same for a float
__device__ __forceinline__ float row16_sum_f(float v)
{
    v += __int_as_float(dpp_or<kRowShr1, 0xf>(0, __float_as_int(v)));
    v += __int_as_float(dpp_or<kRowShr2, 0xf>(0, __float_as_int(v)));
    v += __int_as_float(dpp_or<kRowShr4, 0xf>(0, __float_as_int(v)));
    v += __int_as_float(dpp_or<kRowShr8, 0xf>(0, __float_as_int(v)));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
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

// maximum over lanes 0..15 (the first DPP row), handed to every lane of the wave
__device__ __forceinline__ float row16_max(float v)
{
    v = dpp_max<kRowShr1, 0xf>(v);
    v = dpp_max<kRowShr2, 0xf>(v);
    v = dpp_max<kRowShr4, 0xf>(v);
    v = dpp_max<kRowShr8, 0xf>(v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 15));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_max(double v)
{
    // lanes without a source get their own value back
    const int lo = dpp_or<CTRL, ROW_MASK>(__double2loint(v), __double2loint(v));
    const int hi = dpp_or<CTRL, ROW_MASK>(__double2hiint(v), __double2hiint(v));
    return fmax(v, __hiloint2double(hi, lo));
}

__device__ __forceinline__ double wave_max(double v)
{
    v = dpp_max<kRowShr1, 0xf>(v);
    v = dpp_max<kRowShr2, 0xf>(v);
    v = dpp_max<kRowShr4, 0xf>(v);
    v = dpp_max<kRowShr8, 0xf>(v);
    v = dpp_max<kRowBcast15, 0xa>(v);
    v = dpp_max<kRowBcast31, 0xc>(v);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
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

// One token of the scalar-radius interval pass:  g = e / (du dl), so that gl = g du and gw = g om (om = 1 - x)
// with p^l = (b/S) gl and w = p^u - p^l = ((a-b)/S) gw.
// SPLIT = form 1 - x with the two-float 1/S.  It matters only when some x is close to 1 (the relative
// error of 1 - x is 6e-8 x / (1 - x) without it); rows whose largest probability is at most 1/2 skip it.
template <bool SPLIT = true>
__device__ __forceinline__ void fuse_parts(float e, const FuseRow& r, float& g, float& du, float& om)
{
    om = SPLIT ? fmaf(e, r.nil, fmaf(e, r.nih, 1.0f)) : fmaf(e, r.nih, 1.0f);   // 1 - x
    du = fmaf(e, r.cu, 1.0f);
    const float dl = fmaf(om, r.omb, r.b);
    g = e * __builtin_amdgcn_rcpf(du * dl);
}

template <bool SPLIT = true>
__device__ __forceinline__ void fuse_token(float e, const FuseRow& r, float& gl, float& gw)
{
    float g, du, om;
    fuse_parts<SPLIT>(e, r, g, du, om);
    gl = g * du;
    gw = g * om;
}

// The complement of the width next to gl and gw:  ec = 1 - (p^u - p^l) = (1 - 2 (1-b) x (1-x)) / (du dl)
// (from a b = 1).  The numerator lies in [1/2, 1], so ec keeps its relative accuracy where the width itself
// rounds to 1: with a large radius every p^u_i is close to 1, the widths differ from each other by less
// than an fp32 ulp, and only the sums of ec resolve their standard deviation.
__device__ __forceinline__ void fuse_token_wide(float e, const FuseRow& r, float& gl, float& gw, float& ec)
{
    const float om = fmaf(e, r.nil, fmaf(e, r.nih, 1.0f));        // 1 - x
    const float x = -e * r.nih;
    const float du = fmaf(e, r.cu, 1.0f);
    const float dl = fmaf(om, r.omb, r.b);
    const float rc = __builtin_amdgcn_rcpf(du * dl);
    const float g = e * rc;
    gl = g * du;
    gw = g * om;
    ec = fmaf(-2.0f * r.omb, x * om, 1.0f) * rc;
}

// Tensor-radius mode (Sec. 3.2.3, the Interval Head: r = Softplus(raw)): r = min(kappa Softplus(raw), rmax) in
// fp32.  Softplus(raw) = max(raw, 0) + ln(1 + t), t = e^-|raw|.  With u = fl(1 + t) and d = u - 1 (exact),
// ln(1 + t) = ln(u) + ln(1 + (t - d) / u) = ln(u) + (t - d)(2 - u) to 3e-8 relative: |t - d| is at most half an
// ulp of u and 1/u = 2 - u + d^2/u, so the rounding of 1 + t is put back and small radii (raw << 0, where
// ln(u) alone would be a multiple of 1.2e-7) keep their relative accuracy.  t below half an ulp of 1: u = 1,
// ln(u) = 0 and the correction is t itself.
__device__ __forceinline__ float radius_r(float raw, float kappa, float rmax)
{
    const float t = __builtin_amdgcn_exp2f(-fabsf(raw) * 1.44269504f);
    const float u = 1.0f + t;
    const float d = u - 1.0f;
    const float lg = fmaf(__builtin_amdgcn_logf(u), 0.693147181f, (t - d) * (2.0f - u));
    return fminf(kappa * (fmaxf(raw, 0.f) + lg), rmax);
}

// The same radius in fp64 (one token per row: the reported token's interval).
__device__ __forceinline__ double radius_of(double raw, double kappa, double rmax)
{
    const double sp = raw > 0.0 ? raw + log1p(exp(-raw)) : log1p(exp(raw));
    return fmin(kappa * sp, rmax);
}

// a - 1 = e^r - 1 of a tensor-radius token, r = min(kappa Softplus(raw), rmax); am1_max = e^rmax - 1.
// UNIT (kappa = 1, the Interval Head as the paper defines it): e^Softplus(raw) = 1 + e^raw, so a - 1 = e^raw, capped:
// one exponential, no logarithm, and no cancellation in a - 1 however small the radius is.
template <bool UNIT>
__device__ __forceinline__ float radius_am1(float raw, float kappa, float rmax, float am1_max)
{
    if constexpr (UNIT) return fminf(__builtin_amdgcn_exp2f(fmaf(raw, kLog2eLo, raw * kLog2eHi)), am1_max);
    else return __builtin_amdgcn_exp2f(radius_r(raw, kappa, rmax) * 1.44269504f) - 1.0f;
}

// Tensor-radius token: pl = p^l_i S and w = (p^u_i - p^l_i) S in the units of e, from a - 1 alone.  With
// b = 1/a the lower bound's denominator times a is dl = 1 + (a-1)(1-x) (no cancellation: both terms >= 0), and
//   p^l S = e / dl,   p^u S = a e / du (du = 1 + (a-1) x),   (p^u - p^l) S = (a-1)(a+1) e (1-x) / (du dl),
// so that neither b nor a second reciprocal is needed.
template <bool UNIT>
__device__ __forceinline__ void fuse_token_rad(float e, float raw, const FuseRow& r, float kappa, float rmax,
                                               float am1_max, float& pl, float& w)
{
    const float am1 = radius_am1<UNIT>(raw, kappa, rmax, am1_max);
    const float om = fmaf(e, r.nil, fmaf(e, r.nih, 1.0f));        // 1 - x
    const float x = -e * r.nih;
    const float du = fmaf(am1, x, 1.0f);
    const float dl = fmaf(am1, om, 1.0f);
    const float g = e * __builtin_amdgcn_rcpf(du * dl);
    pl = g * du;
    w = (am1 * (am1 + 2.0f)) * (g * om);
}

// The same with the complement of the width (see fuse_token_wide), in the same units:
// ec = 1 - (p^u_i - p^l_i) = (a - 2 (a-1) x (1-x)) / (du dl).
template <bool UNIT>
__device__ __forceinline__ void fuse_token_rad_wide(float e, float raw, const FuseRow& r, float kappa, float rmax,
                                                    float am1_max, float& pl, float& w, float& ec)
{
    const float am1 = radius_am1<UNIT>(raw, kappa, rmax, am1_max);
    const float om = fmaf(e, r.nil, fmaf(e, r.nih, 1.0f));        // 1 - x
    const float x = -e * r.nih;
    const float du = fmaf(am1, x, 1.0f);
    const float dl = fmaf(am1, om, 1.0f);
    const float rc = __builtin_amdgcn_rcpf(du * dl);
    const float g = e * rc;
    pl = g * du;
    w = (am1 * (am1 + 2.0f)) * (g * om);
    ec = fmaf(-2.0f * am1, x * om, am1 + 1.0f) * rc;
}

// The two with the choice made at run time (uniform over a launch).
struct RadiusMode { bool unit; float kappa, rmax, am1_max; };
__device__ __forceinline__ RadiusMode radius_mode(const RowArgs& A)
{
    return {A.kappa == 1.0, (float)A.kappa, (float)A.rmax, (float)expm1(A.rmax)};
}
__device__ __forceinline__ void fuse_token_rad(float e, float raw, const FuseRow& r, const RadiusMode& m, float& pl,
                                               float& w)
{
    if (m.unit) fuse_token_rad<true>(e, raw, r, m.kappa, m.rmax, m.am1_max, pl, w);
    else fuse_token_rad<false>(e, raw, r, m.kappa, m.rmax, m.am1_max, pl, w);
}
__device__ __forceinline__ void fuse_token_rad_wide(float e, float raw, const FuseRow& r, const RadiusMode& m,
                                                    float& pl, float& w, float& ec)
{
    if (m.unit) fuse_token_rad_wide<true>(e, raw, r, m.kappa, m.rmax, m.am1_max, pl, w, ec);
    else fuse_token_rad_wide<false>(e, raw, r, m.kappa, m.rmax, m.am1_max, pl, w, ec);
}

// Vocabularies of at most this many tokens take fp64 token arithmetic (see fuse_sums_tiny, dro_row_tiny_kernel).
constexpr int kTinyVocab = 64;

// Per-row scalars of the quantifier from the five sums (fp64, one lane).
struct RowScore { double alpha_l, alpha_u, omega, sigma, score; };

// How a row's interval sums are to be read (RowStats::mode).
constexpr float kSumsFull = 0.f;         // all five sums
constexpr float kSumsWidthOnly = 1.f;    // the caps are known to be inactive; only sum gw, sum gw^2 were accumulated
constexpr float kSumsComplement = 2.f;   // caps inactive, every width above 1/2: q[1] = sum ec, q[3] = sum ec^2
constexpr float kSumsDirect = 3.f;       // all five sums, of p^l_i and p^u_i - p^l_i themselves (no row factor)
constexpr float kSumsFlatPending = 8.f;  // added to the above: a flat row that flatrow_kernel has still to redo

// The sums arrive shifted: s = { sum (gl - kl), sum (gw - kw), sum (gl - kl)^2, sum (gw - kw)^2,
// sum (gl - kl)(gw - kw) } over the V tokens of the row, where (kl, kw) are the values of one of the row's own
// tokens.  Sums and sums of squares taken about such a point lose at most a factor V of fp64's 1e-16 when the
// squared mean is subtracted, however small the spread is against the mean (a row of equal logits has spread 0
// and mean > 0: about the origin the difference of the two moments is rounding noise of relative size 1e-8
// after the square root, which Omega ~ V then multiplies).  Pass kl = kw = 0 for plain sums.
__device__ __forceinline__ RowScore finish_score(const double* s, double S, float mode, const RowArgs& A,
                                                 double kl, double kw)
{
    // p^l_i = Bc gl_i and p^u_i - p^l_i = Wc gw_i (tensor-radius mode: the per-token factors are already
    // inside gl and gw)
    const double V = (double)A.V;
    if (mode >= kSumsFlatPending) mode -= kSumsFlatPending;        // marked, not (yet) redone: the sums are valid as they are
    if (mode == kSumsComplement) {
        // s[1], s[3]: sums of (ec_i - kw) and its square, ec_i = 1 - delta_i:  Omega = V - sum ec,
        // Var(delta) = Var(ec), the latter taken among the small ec_i themselves instead of among numbers that
        // all round to 1
        RowScore o;
        o.alpha_l = 1.0; o.alpha_u = 1.0;
        o.omega = V - (s[1] + V * kw);
        o.sigma = sqrt(fmax(0.0, s[3] - s[1] * s[1] / V) / V);
        o.score = o.omega * o.sigma;
        return o;
    }
    const bool capless = mode == kSumsWidthOnly;
    const bool direct = mode == kSumsDirect;
    const double Bc = direct ? 1.0 : (A.radius ? 1.0 : A.b) / S, Wc = direct ? 1.0 : (A.radius ? 1.0 : A.a - A.b) / S;
    const double sum_gl = s[0] + V * kl, sum_gw = s[1] + V * kw;
    // S_l <= 1 <= S_u holds for every radius (p^l_i <= x_i <= p^u_i token by token); the computed sums carry ~1e-7
    // of fp32 token arithmetic and may land on the wrong side of 1 for a one-hot row, which a cap of exactly 1
    // would turn into a spurious scaling
    const double Sl = fmin(1.0, Bc * sum_gl), Su = fmax(1.0, Bc * sum_gl + Wc * sum_gw);
    RowScore o;
    o.alpha_l = 1.0; o.alpha_u = 1.0;
    if (A.normalize && !capless) {
        o.alpha_l = fmin(1.0, A.cap_lo / Sl);
        o.alpha_u = fmax(1.0, A.cap_hi / Su);
    }
    // delta_i = alpha_u p^u_i - alpha_l p^l_i = alpha_u w_i + (alpha_u - alpha_l) p^l_i = cw gw_i + cl gl_i:
    // both coefficients are >= 0, so Omega is a sum of non-negative terms; the spread is that of
    // delta_i - (cw kw + cl kl) = cw (gw_i - kw) + cl (gl_i - kl).
    const double cw = o.alpha_u * Wc, cl = (o.alpha_u - o.alpha_l) * Bc;
    o.omega = cw * sum_gw + (capless ? 0.0 : cl * sum_gl);
    const double T1 = cw * s[1] + cl * s[0];
    const double T2 = cw * cw * s[3] + 2.0 * cw * cl * s[4] + cl * cl * s[2];
    o.sigma = sqrt(fmax(0.0, T2 - T1 * T1 / V) / V);
    o.score = o.omega * o.sigma;
    return o;
}

// The accept test of a drafted token in the log domain, fp64 (Algorithm 1, "Cloud verification"):
//   ln p_x = cx - n ln2 - ln S,  ln q_x = tx - nt ln2 - ln Z;  accepted iff ln u < min(0, ln q_x - ln p_x).
// Returns whether the token is rejected.
__device__ __forceinline__ bool reject_exact(float cx, float tx, float u, float n, float nt, double S, double Z)
{
    const double lp = ((double)cx - (double)n * kLn2) - log(S);
    const double lq = ((double)tx - (double)nt * kLn2) - log(Z);
    const double lnu = log((double)u);                             // log(0) = -inf: always accepted
    return !(lnu < fmin(0.0, lq - lp));
}

// The same test in fp32 with the hardware logarithm, for the streaming kernel, where every wave of a row evaluates
// it: 1 = accepted, 0 = rejected, -1 = too close to call (then reject_exact decides).  The fp32 evaluation is off by
// at most ~3e-7 (1 + the sum of the magnitudes of its terms): a hardware logarithm good to an ulp, a handful of
// roundings at 6e-8; the guard band is thirty times that, and a row falls inside it about once in a few thousand.
// Anything that is not a number ends up in the band.
__device__ __forceinline__ int accept_quick(float cx, float tx, float u, float n, float nt, float S, float Z)
{
    const float lS = __builtin_amdgcn_logf(S), lZ = __builtin_amdgcn_logf(Z);   // base 2
    const float lu = __builtin_amdgcn_logf(u);
    const float d = tx - cx, dn = nt - n;
    const float ell = fmaf(-(dn + (lZ - lS)), 0.693147181f, d);   // ln q_x - ln p_x
    const float margin = fminf(0.f, ell) - lu * 0.693147181f;     // > 0: accepted
    const float guard = 1e-5f * (1.f + fabsf(d) + fabsf(dn) + fabsf(lZ) + fabsf(lS) + fabsf(lu));
    if (u == 0.f && ell > -INFINITY) return 1;                     // ln 0 = -inf lies below every finite bound
    if (margin > guard) return 1;
    if (margin < -guard) return 0;
    return -1;
}

// One row's outputs from its statistics, in fp64 (Eq. uncertainty_score; Algorithm 1's threshold and verification
// steps): score, flag, the reported token's interval, the accept test in the log domain.  xid = the reported
// token (-1: the arg-max token, whose logit is st.mc), cx / tx / rawx = its centre logit, verifier logit and raw
// radius, u = the row's uniform for the accept test.  Returns whether the drafted token is rejected.
__device__ __forceinline__ bool finish_row(const RowArgs& A, int64_t row, const RowStats& st, float cx, float tx,
                                           float rawx, float u, bool do_q, bool do_v)
{
    const double S = st.S;
    const float n = st.n;
    if (do_q) {
        double q[5] = {st.q[0], st.q[1], st.q[2], st.q[3], st.q[4]};
        // The token above 1/2 of a row whose caps can be active, once more in fp64.  Where a cap is active
        // Omega = alpha_u S_u - alpha_l S_l is a small difference of numbers near 1, and on a nearly one-hot row S_l is
        // little more than that token's lower bound: its fp32 evaluation in the streaming kernel (a hardware reciprocal
        // of a rounded product and three more roundings) leaves ~2e-7 of it, the whole absolute tolerance of an Omega of
        // 0.01 (a seeded random case: 2.04e-7 off).  At most one token of a row is above 1/2: the row's largest, whose
        // wave has the row's reference, so its e and the fp32 values that the scalar-radius pass has added to the sums
        // can be formed again here, by the same instructions, and exchanged for the fp64 values.  (Plain sums only:
        // such a row is not flat.  Tensor-radius, wide-radius and tiny-vocabulary rows come from other passes.)
        // (the call's constants through an empty asm: what is derived from them here is otherwise formed at the top of
        // the calling kernel and kept -- in the streaming kernel: spilled -- through its row loop)
        double fa = A.a, fb = A.b;
        int fv = A.V;
        asm volatile("" : "+s"(fa), "+s"(fb), "+s"(fv));
        if (st.mode == kSumsFull && A.normalize && !A.radius && fv > kTinyVocab && fa < 3.0 * (double)fv &&
            st.kl == 0.0 && st.kw == 0.0) {
            const float etop = exp2_ref(st.mc, n == -INFINITY ? 0.f : n);
            if ((double)etop > 0.5 * S) {
                const double ed = (double)etop, invS = 1.0 / S;
                const double x = ed * invS, om = fmax(0.0, S - ed) * invS;      // 1 - x from the sum of the other tokens
                const double du = 1.0 + (fa - 1.0) * x, dl = fb + (1.0 - fb) * om;
                const double gl = ed / dl, gw = gl * om / du;
                float g, duf, omf;
                fuse_parts<true>(etop, fuse_row(S, fa, fb), g, duf, omf);
                const double glf = (double)(g * duf), gwf = (double)(g * omf);
                q[0] += gl - glf;
                q[1] += gw - gwf;
                q[2] += gl * gl - glf * glf;
                q[3] += gw * gw - gwf * gwf;
                q[4] += gl * gw - glf * gwf;
            }
        }
        const RowScore rs = finish_score(q, S, st.mode, A, st.kl, st.kw);
        if (A.omega) A.omega[row] = (float)rs.omega;
        if (A.sigma) A.sigma[row] = (float)rs.sigma;
        if (A.score) A.score[row] = (float)rs.score;
        if (A.flags) A.flags[row] = (uint8_t)(rs.score > A.tau);
        if (A.p_lo || A.p_mid || A.p_hi) {
            // e_x exactly as the streaming kernel summed it into S (the arg-max token, the only one whose
            // probability can approach 1, sits in a wave whose reference is n), so that S - e_x is the
            // sum of the other tokens to fp64 rounding and 1 - x keeps its relative accuracy as x -> 1:
            // the lower bound's denominator b + (1-b)(1-x) is that small number when b is small too.
            const double ex = (double)exp2_ref(cx, n == -INFINITY ? 0.f : n);
            const double x = ex / S, omx = fmax(0.0, S - ex) / S;
            double a = A.a, b = A.b;
            if (A.radius) {
                // the reported token's own radius (the launcher supplies ids in this mode)
                const double r = radius_of((double)rawx, A.kappa, A.rmax);
                a = exp(r); b = exp(-r);
            }
            if (A.p_mid) A.p_mid[row] = (float)x;
            if (A.p_lo) A.p_lo[row] = (float)(rs.alpha_l * b * x / (b + (1.0 - b) * omx));
            if (A.p_hi) A.p_hi[row] = (float)(rs.alpha_u * a * x / (1.0 + (a - 1.0) * x));
        }
    }
    bool rej = false;
    if (do_v) {
        rej = reject_exact(cx, tx, u, n, st.nt, S, st.Z);
        if (A.accept) A.accept[row] = (uint8_t)(!rej);
        if (A.row_id && !rej) A.row_id[row] = -1;
    }
    return rej;
}

// The rows of a window that spans workgroups meet in one 64-bit word of caller memory, which needs no
// initialisation and carries everything the window's outputs need, so that no other memory has to be made visible
// between workgroups:  [63:33] the launch's tag (RowArgs::tag, never zero, different for every launch of the process: a
// word with another tag -- what an earlier call left behind, or whatever the memory held before -- is a fresh one),
// [32:25] rows arrived, [24:17] offset of the first rejected row so far (255: none), [16:0] that row's draw.
// A run of `rows` consecutive rows of the window that one workgroup has finished arrives with one call: its rows'
// first rejected offset in the window and that row's draw (id = -1: all accepted).  The call that completes the
// window returns true with the window's first rejected offset (-1: none) and its draw.
constexpr int kMaxCountedWindow = 255;
__device__ __forceinline__ bool window_arrive(unsigned long long* p, uint32_t tag, int rows, int off, int id, int len,
                                              int& first, int& draw)
{
    const unsigned long long t31 = (unsigned long long)(tag & 0x7fffffffu);
    // The first exchange assumes a fresh word, which window_claim has normally left there at the start of the
    // kernel: the trip to memory and back that reading the word first would cost is the tail of the kernel.
    unsigned long long seen = (t31 << 33) | (0xffull << 17);
    for (;;) {
        const unsigned long long cur = (seen >> 33) == t31 ? seen : ((t31 << 33) | (0xffull << 17));
        const unsigned long long count = ((cur >> 25) & 0xffull) + (unsigned long long)rows;
        unsigned long long f = (cur >> 17) & 0xffull, d = cur & 0x1ffffull;
        if (id >= 0 && (unsigned long long)off < f) { f = (unsigned long long)off; d = (unsigned long long)id & 0x1ffffull; }
        const unsigned long long next = (t31 << 33) | (count << 25) | (f << 17) | d;
        const unsigned long long prev = atomicCAS(p, seen, next);
        if (prev == seen) {
            first = f == 0xffull ? -1 : (int)f;
            draw = (int)d;
            if (count != (unsigned long long)len) return false;
            // complete: hand the word back (a replay of this launch from a captured graph carries the same tag)
            __hip_atomic_store(p, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return true;
        }
        seen = prev;                                               // another row of the window got in between
    }
}

// Makes a window's word a fresh one of this launch ahead of its rows' arrivals (an optimisation only: window_arrive
// copes with whatever it finds).
// `seen` = what the caller has read in the word (an atomic load issued early, so that its trip to memory is over).
// One exchange whose outcome is not awaited: if it fails, another workgroup has claimed the word or arrived in it in
// the meantime, and the word is what it should be.
__device__ __forceinline__ void window_claim(unsigned long long* p, uint32_t tag, unsigned long long seen)
{
    const unsigned long long t31 = (unsigned long long)(tag & 0x7fffffffu), fresh = (t31 << 33) | (0xffull << 17);
    if ((seen >> 33) != t31) (void)atomicCAS(p, seen, fresh);
}

// Compute units of the current device (asked once per device, then cached; the cache is a relaxed atomic per device:
// two threads that ask at once both write the same number).
inline int compute_units()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    static std::atomic<int> cache[64];
    int cus = cache[dev].load(std::memory_order_relaxed);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        cache[dev].store(cus, std::memory_order_relaxed);
    }
    return cus;
}

}  // namespace
}  // namespace ciar
