// gfx950 kernels of the CIAR quantify + verify pass.
//
// One workgroup owns one row (one drafted token position).  The centre row c and the verifier
// row t are fetched once with 16-byte loads, interleaved over the workgroup so that every load
// instruction of a wave covers 1 KiB of consecutive memory, and stay in registers for the whole
// life of the workgroup: the InterFuse bounds need the partition sum S of the complete row
// before the first bound can be formed (App. "Proof of Interval Validity": S appears in every
// denominator), so the row has to be resident between the statistics pass and the interval pass.
// Nothing V-wide is ever written back.
//
// Per row:
//   A  max of c and of t                                   (max-trick)
//   B  e_i = exp(c_i - max c) kept in registers, S = sum e_i;  Z = sum exp(t_i - max t)
//   C  InterFuse for a scalar radius r, a = e^r, b = e^-r, x_i = e_i / S:
//        p^u_i = a x_i / (1 + (a-1) x_i),   p^l_i = b x_i / (1 - (1-b) x_i)
//      with one reciprocal of the product of the two denominators, accumulated as the lower
//      bound p^l_i and the raw width w_i = p^u_i - p^l_i = (a-b) x_i (1-x_i) / (du_i dl_i).
//      Five sums per row (sum p^l, sum w and the three second moments, all taken about the
//      values of the uniform row so that nearly flat rows do not cancel) give, after the
//      0.99 / 1.01 caps alpha_l, alpha_u are known,
//        delta_i = alpha_u w_i + (alpha_u - alpha_l) p^l_i,
//        Omega   = sum delta_i,   Sigma^2 = (sum (delta_i - mean)^2) / V,   U = Omega * Sigma
//      without a second sweep over the row.                 (Eq. uncertainty_score)
//   D  flag = U > tau; interval of the drafted token; accept test in the log domain (fp64,
//      one lane):  ln u < min(0, ln q_x - ln p_x)
//   E  rejected rows only (workgroup-uniform branch): res_i = max(0, q_i - p_i), inverse-CDF
//      draw in token order from a workgroup-wide prefix sum.
//
// Sums over the row are accumulated per lane in fp32 and combined across lanes and waves in
// fp64 in a fixed order, so results are deterministic and the per-row scalars carry ~1e-8
// relative error.
#include "ciar_internal.h"

#include <limits.h>
#include <math.h>

namespace ciar {
namespace {

// log2(e) split so that the low part is positive: d * hi + d * lo stays -inf for d = -inf.
constexpr float  kLog2eHi = 1.44269490242004394531f;   // largest float below log2(e)
constexpr float  kLog2eLo = 1.384689195e-7f;           // log2(e) - kLog2eHi

__device__ __forceinline__ float bits_f(uint32_t u) { return __uint_as_float(u); }

// 16 bytes as loaded: a native vector type, so it can be read through an address-space pointer.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// exp(x - m) for x <= m.  The difference d = x - m is formed first: it is exact for logits near the
// maximum and its rounding error shrinks with |d|, so the tokens that carry the mass get full
// precision and the row maximum maps to exactly 1.  d * log2(e) uses the two-term constant.
__device__ __forceinline__ float exp_shifted(float x, float m)
{
    const float d = x - m;
    return __builtin_amdgcn_exp2f(fmaf(d, kLog2eHi, d * kLog2eLo));
}

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
};

// ---- wave and workgroup reductions (fixed order: deterministic) ----------------------------
//
// Wave-level reductions use DPP row shifts and row broadcasts: they run on the vector ALU at full
// rate, whereas a shuffle (ds_bpermute) goes through the LDS crossbar and costs ~5x more per step.
// Pattern (wave64 = 4 rows of 16 lanes): row_shr 1, 2, 4, 8 leave each row's total in its lane 15;
// row_bcast:15 adds it into the next row (rows 1 and 3), row_bcast:31 adds lane 31 into rows 2
// and 3; lane 63 then holds the wave total, which readlane hands to every lane.

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

__device__ __forceinline__ double wave_sum(double v)
{
    v = dpp_add<kRowShr1, 0xf>(v);
    v = dpp_add<kRowShr2, 0xf>(v);
    v = dpp_add<kRowShr4, 0xf>(v);
    v = dpp_add<kRowShr8, 0xf>(v);
    v = dpp_add<kRowBcast15, 0xa>(v);
    v = dpp_add<kRowBcast31, 0xc>(v);
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

// inclusive prefix sum over the 64 lanes (same steps, without the final broadcast)
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

// All threads end up with the workgroup-wide sums of v[0..NV).  smem: NW*NV doubles.
template <int NW, int NV>
__device__ __forceinline__ void block_sum(double (&v)[NV], double* smem, int lane, int wave)
{
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = wave_sum(v[i]);
    __syncthreads();
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) smem[wave * NV + i] = v[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += smem[w * NV + i];
        v[i] = s;
    }
}

template <int NW>
__device__ __forceinline__ float block_max(float m, double* smem, int lane, int wave)
{
    m = wave_max(m);
    float* f = reinterpret_cast<float*>(smem);
    __syncthreads();
    if (lane == 0) f[wave] = m;
    __syncthreads();
    float r = f[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = fmaxf(r, f[w]);
    return r;
}

// ---- per-token InterFuse arithmetic, shared by the row kernel and the dense export ----------

// Constants of one row for a scalar radius.  Units: e_i = exp(c_i - max c), S = sum e_i.
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
__device__ __forceinline__ void fuse_token(float e, const FuseRow& r, float& gl, float& gw)
{
    const float om = fmaf(e, r.nil, fmaf(e, r.nih, 1.0f));        // 1 - x
    const float du = fmaf(e, r.cu, 1.0f);
    const float dl = fmaf(om, r.omb, r.b);
    const float g = e * __builtin_amdgcn_rcpf(du * dl);
    gl = g * du;
    gw = g * om;
}

// Per-row scalars of the quantifier from the five centred sums (fp64, one lane).
struct RowScore { double alpha_l, alpha_u, omega, sigma, score; };

__device__ __forceinline__ RowScore finish_score(const double (&s)[5], double S, const RowArgs& A)
{
    // s = { sum gl, sum gw, sum gl^2, sum gw^2, sum gl gw } over the V tokens of the row
    const double V = (double)A.V;
    const double Bc = A.b / S, Wc = (A.a - A.b) / S;
    const double Sl = Bc * s[0], Su = Sl + Wc * s[1];
    RowScore o;
    o.alpha_l = 1.0; o.alpha_u = 1.0;
    if (A.normalize) {
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

// Waves per SIMD the register allocation aims for.  One row at a time is resident (the verifier row
// is consumed before the centre row is fetched into the same registers): EPT floats plus ~50 working
// registers, capped at 4 waves (more buys nothing for a kernel that streams 64 KiB per workgroup).
template <typename T, int THREADS, int NVEC>
constexpr int target_waves()
{
#ifdef XP_WAVES
    return XP_WAVES < THREADS / 256 ? THREADS / 256 : XP_WAVES;
#endif
    constexpr int regs = NVEC * Elt<T>::kPerVec + 56;
    constexpr int fit = 512 / regs;
    constexpr int lo = THREADS / 256;                 // waves per SIMD one workgroup needs
    return fit < lo ? lo : (fit > 4 ? 4 : fit);
}

// Pass C for one lane: the five InterFuse sums over the lane's tokens.
// MASKED = the row does not fill the tile: chunks past the end are skipped (padding inside the last
// chunk has e = 0 and adds exactly nothing).
template <int THREADS, int NVEC, int EPV, bool MASKED>
__device__ __forceinline__ void fuse_sums(const float (&e)[NVEC * EPV], const FuseRow& fr, int V,
                                          double (&q5)[5])
{
    // The five sums run in fp64 from the first add (fp64 adds and FMAs issue at the fp32 rate on this
    // chip).  One token can hold almost all of sum(gl), and the variance is a difference of second
    // moments that would cancel in fp32 on nearly flat rows; in fp64 neither needs a centring trick.
    double a0[2] = {0.0, 0.0}, a1[2] = {0.0, 0.0}, a2[2] = {0.0, 0.0}, a3[2] = {0.0, 0.0}, a4[2] = {0.0, 0.0};
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        if (MASKED && j * THREADS * EPV >= V) continue;            // uniform: the chunk holds no token
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float gl, gw;
            fuse_token(e[j * EPV + k], fr, gl, gw);                // padding has e = 0: gl = gw = 0
            const double dl = (double)gl, dw = (double)gw;
            a0[k & 1] += dl;
            a1[k & 1] += dw;
            a2[k & 1] = fma(dl, dl, a2[k & 1]);
            a3[k & 1] = fma(dw, dw, a3[k & 1]);
            a4[k & 1] = fma(dl, dw, a4[k & 1]);
        }
        __builtin_amdgcn_sched_barrier(0);                         // one vector at a time: bounded working set
    }
    q5[0] = a0[0] + a0[1];
    q5[1] = a1[0] + a1[1];
    q5[2] = a2[0] + a2[1];
    q5[3] = a3[0] + a3[1];
    q5[4] = a4[0] + a4[1];
}

template <typename T>
__device__ __forceinline__ float load_logit(const T* row, int i)
{
    if constexpr (sizeof(T) == 4) return reinterpret_cast<const float*>(row)[i];
    else return bits_f((uint32_t)reinterpret_cast<const uint16_t*>(row)[i] << 16);
}

template <typename T, int THREADS, int NVEC, bool DO_Q, bool DO_V>
__global__ __launch_bounds__(THREADS)
__attribute__((amdgpu_waves_per_eu(target_waves<T, THREADS, NVEC>())))
void row_kernel(const RowArgs A)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec;
    constexpr int EPT = NVEC * EPV;
    constexpr int NW = THREADS / 64;
    constexpr int CHUNK = THREADS * EPV;            // tokens covered by one load instruction of the workgroup
    constexpr int EB = NVEC > 8 ? 8 : NVEC;         // vectors of each row in flight per lane in the residual pass

    __shared__ double smem[NW * (NVEC > 5 ? NVEC : 5) + NW];
    __shared__ int    smem_i[NW * 2 + 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = A.V;
    const bool partial = V != NVEC * CHUNK;                        // uniform: the row does not fill the tile
    const int last_vec = (V + EPV - 1) / EPV - 1;

    // Rows live in global memory (address space 1): say so, or the loads are emitted as flat ones.
    // Vector indices past the end of the row are clamped to its last vector, so every lane loads
    // valid memory unconditionally; tokens that do not exist are set to -inf afterwards.
    using gbytes = const __attribute__((address_space(1))) char*;
    using gvec = const __attribute__((address_space(1))) u32x4*;
    const T* crow = static_cast<const T*>(A.draft) + row * A.stride;
    const T* trow = DO_V ? static_cast<const T*>(A.target) + row * A.stride : nullptr;
    // vector j of this lane: uniform row base + 32-bit byte offset (one VGPR per address)
    auto load_vec_at = [&](const T* base, int j, int t) -> u32x4 {
        const uint32_t off = (uint32_t)min(j * THREADS + t, last_vec) * 16u;
        return *(gvec)((gbytes)base + off);
    };
    auto load_vec = [&](const T* base, int j) -> u32x4 { return load_vec_at(base, j, tid); };

    u32x4 raw[NVEC];                                               // landing registers: t first, then c

    // ---- T: verifier row statistics (max, Z); the row is not kept ---------------------------------
    int xid = -1;
    float cx = 0.f, tx = 0.f, ua = 0.f, ur = 0.f;
    float mt = -INFINITY;
    double sz[2] = {0.0, 0.0};                                     // lane partials of S and Z
    if constexpr (DO_V) {
#pragma unroll
        for (int j = 0; j < NVEC; ++j) raw[j] = load_vec(trow, j);
    }
    if (tid == 0) {                                                // the row's scalars and the drafted token's logits
        if (A.ids) {
            xid = A.ids[row];
            xid = xid < 0 ? 0 : (xid >= V ? V - 1 : xid);
            cx = load_logit(crow, xid);
        }
        if constexpr (DO_V) {
            tx = load_logit(trow, xid);
            ua = A.u_accept[row];
            ur = A.u_resample[row];
        }
    }
    if constexpr (DO_V) {
        if (partial) {
#pragma unroll
            for (int j = 0; j < NVEC; ++j) E::mask_tail(raw[j], (j * THREADS + tid) * EPV, V);
        }
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            float tv[EPV];
            E::unpack(raw[j], tv);
#pragma unroll
            for (int k = 0; k < EPV; ++k) mt = fmaxf(mt, tv[k]);
        }
        mt = block_max<NW>(mt, smem, lane, wave);
        float zacc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            float tv[EPV];
            E::unpack(raw[j], tv);
#pragma unroll
            for (int k = 0; k < EPV; ++k) zacc[k & 3] += exp_shifted(tv[k], mt);
            __builtin_amdgcn_sched_barrier(0);
        }
        sz[1] = (double)((zacc[0] + zacc[1]) + (zacc[2] + zacc[3]));
        __builtin_amdgcn_sched_barrier(0);                         // t is dead: its registers take the centre row
    }

    // ---- A + B: centre row: max, e_i = exp(c_i - max), S ----------------------------------------------
    {
#pragma unroll
        for (int j = 0; j < NVEC; ++j) raw[j] = load_vec(crow, j);
        if (partial) {
#pragma unroll
            for (int j = 0; j < NVEC; ++j) E::mask_tail(raw[j], (j * THREADS + tid) * EPV, V);
        }
    }
    float e[EPT];
#pragma unroll
    for (int j = 0; j < NVEC; ++j) E::unpack(raw[j], &e[j * EPV]);
    float mc = e[0];
#pragma unroll
    for (int i = 1; i < EPT; ++i) mc = fmaxf(mc, e[i]);
    mc = block_max<NW>(mc, smem, lane, wave);
    {
        // S is accumulated in fp64 from the first add: on a nearly one-hot row the bounds of the top
        // token react to a relative error in S about five times over, and adding small terms to an
        // fp32 partial sum that already holds 1.0 would cost 1e-7.
        double sacc[2] = {0.0, 0.0};
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
#pragma unroll
            for (int k = 0; k < EPV; ++k) {
                e[j * EPV + k] = exp_shifted(e[j * EPV + k], mc);
                sacc[k & 1] += (double)e[j * EPV + k];
            }
            __builtin_amdgcn_sched_barrier(0);                     // keep the working set to one vector at a time
        }
        sz[0] = sacc[0] + sacc[1];
    }
    block_sum<NW, 2>(sz, smem, lane, wave);
    const double S = sz[0], Z = sz[1];
    const double mcd = (double)mc, mtd = (double)mt;

    // ---- D1: accept test (one lane, fp64, log domain) ----------------------------------------------------
    if constexpr (DO_V) {
        if (tid == 0) {
            const double lp = ((double)cx - mcd) - log(S);
            const double lq = ((double)tx - mtd) - log(Z);
            const double ell = lq - lp;
            const double lnu = log((double)ua);                    // log(0) = -inf: always accepted
            const int rej = !(lnu < fmin(0.0, ell));
            if (A.accept) A.accept[row] = (uint8_t)(!rej);
            if (!rej && A.row_id) A.row_id[row] = -1;
            smem_i[NW * 2] = rej;                                  // read by everyone after the next barrier
            smem_i[NW * 2 + 1] = __float_as_int(ur);
        }
    }

    // ---- C + D2: InterFuse sums, score, flag and the drafted token's interval ------------------------
    if constexpr (DO_Q) {
        const FuseRow fr = fuse_row(S, A.a, A.b);
        double q5[5];
        if (partial) fuse_sums<THREADS, NVEC, EPV, true>(e, fr, V, q5);
        else         fuse_sums<THREADS, NVEC, EPV, false>(e, fr, V, q5);
        block_sum<NW, 5>(q5, smem, lane, wave);
        if (tid == 0) {
            const RowScore rs = finish_score(q5, S, A);
            if (A.omega) A.omega[row] = (float)rs.omega;
            if (A.sigma) A.sigma[row] = (float)rs.sigma;
            if (A.score) A.score[row] = (float)rs.score;
            if (A.flags) A.flags[row] = (uint8_t)(rs.score > A.tau);
            if (A.p_lo || A.p_mid || A.p_hi) {
                // the reported token: the drafted one, or the arg-max (e = 1) when no ids are given
                const double ex = exp((double)(xid >= 0 ? cx : mc) - mcd);
                const double x = ex / S;
                if (A.p_mid) A.p_mid[row] = (float)x;
                if (A.p_lo) A.p_lo[row] = (float)(rs.alpha_l * A.b * x / (1.0 + (A.b - 1.0) * x));
                if (A.p_hi) A.p_hi[row] = (float)(rs.alpha_u * A.a * x / (1.0 + (A.a - 1.0) * x));
            }
        }
    }

    // ---- E: residual resample of a rejected row (workgroup-uniform branch) -----------------------------
    // res_i = max(0, q_i - p_i).  Self-contained on purpose: both rows are fetched again (they were just
    // read, so this comes from cache) and e_i, exp(t_i - max t) are recomputed bit-identically, so that
    // no register of the main path has to stay alive for a branch only ~1 row in 8 takes.
    if constexpr (DO_V) {
        __syncthreads();
        const int rejected = smem_i[NW * 2];
        if (rejected && A.row_id) {
            const double u_res = (double)__int_as_float(smem_i[NW * 2 + 1]);
            const double invS = 1.0 / S, invZ = 1.0 / Z;
            // The lane index is laundered through an empty asm so that the addresses of this rare branch
            // are formed here instead of being kept alive (and spilled) across the whole main path.
            int tid_e = tid;
            asm volatile("" : "+v"(tid_e));
            // residuals of one 16-byte vector of each row
            auto residuals = [&](u32x4 cr, u32x4 tr, int j, float (&r)[EPV]) {
                if (partial) {
                    E::mask_tail(cr, (j * THREADS + tid_e) * EPV, V);
                    E::mask_tail(tr, (j * THREADS + tid_e) * EPV, V);
                }
                float cv[EPV], tv[EPV];
                E::unpack(cr, cv);
                E::unpack(tr, tv);
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    const double q = (double)exp_shifted(tv[k], mt) * invZ;
                    const double p = (double)exp_shifted(cv[k], mc) * invS;
                    r[k] = (float)fmax(q - p, 0.0);
                }
            };
            // E1: workgroup totals of the residual over each chunk of CHUNK tokens
#pragma unroll
            for (int b0 = 0; b0 < NVEC; b0 += EB) {
                u32x4 cb[EB], tb[EB];
#pragma unroll
                for (int jj = 0; jj < EB; ++jj) {
                    cb[jj] = load_vec_at(crow, b0 + jj, tid_e);
                    tb[jj] = load_vec_at(trow, b0 + jj, tid_e);
                }
#pragma unroll
                for (int jj = 0; jj < EB; ++jj) {
                    float r[EPV];
                    residuals(cb[jj], tb[jj], b0 + jj, r);
                    float s = 0.f;
#pragma unroll
                    for (int k = 0; k < EPV; ++k) s += r[k];
                    const double ws = wave_sum((double)s);
                    if (lane == 0) smem[wave * NVEC + b0 + jj] = ws;
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            __syncthreads();
            double R = 0.0;
#pragma unroll
            for (int j = 0; j < NVEC; ++j) {
#pragma unroll
                for (int w = 0; w < NW; ++w) R += smem[w * NVEC + j];
            }
            int cand = INT_MAX, lastpos = -1;
            if (R > 0.0) {
                // chunk that holds the crossing of u * R (token order = chunk order, then lane order)
                const double thr = u_res * R;
                int jstar = -1, jlast = 0;
                double before = 0.0, run = 0.0;
#pragma unroll
                for (int j = 0; j < NVEC; ++j) {
                    double tot = 0.0;
#pragma unroll
                    for (int w = 0; w < NW; ++w) tot += smem[w * NVEC + j];
                    if (jstar < 0 && run + tot > thr) { jstar = j; before = run; }
                    if (tot > 0.0) jlast = j;
                    if (jstar < 0) run += tot;
                }
                if (jstar < 0) { jstar = jlast; before = run; }    // unreachable for u < 1; keeps the draw valid
                // E2: the lane's residuals inside that chunk, recomputed exactly as in E1
                float r[EPV];
                residuals(load_vec_at(crow, jstar, tid_e), load_vec_at(trow, jstar, tid_e), jstar, r);
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < EPV; ++k) s += r[k];
                const double incl = wave_scan((double)s);
                if (lane == 63) smem[NW * NVEC + wave] = incl;
                __syncthreads();
                double cum = before + (incl - (double)s);
#pragma unroll
                for (int w = 0; w < NW; ++w)
                    if (w < wave) cum += smem[NW * NVEC + w];
                // smallest token of the chunk whose inclusive running sum exceeds u * R; tokens without
                // residual mass cannot be drawn; lastpos covers a crossing lost to rounding at the chunk end
                const int base = (jstar * THREADS + tid_e) * EPV;
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    cum += (double)r[k];
                    if (r[k] > 0.f) {
                        lastpos = base + k;
                        if (cum > thr && cand == INT_MAX) cand = base + k;
                    }
                }
            } else {
                // every residual rounded to zero (q == p to working precision): the draw degenerates
                // to the lowest-index arg-max of q; this path is practically never taken
                for (int i = tid; i < V; i += THREADS)
                    if (load_logit(trow, i) == mt) { cand = i; break; }
            }
            cand = wave_min_i(cand);
            lastpos = wave_max_i(lastpos);
            if (lane == 0) { smem_i[wave * 2] = cand; smem_i[wave * 2 + 1] = lastpos; }
            __syncthreads();
            if (tid == 0) {
                int c0 = smem_i[0], l0 = smem_i[1];
#pragma unroll
                for (int w = 1; w < NW; ++w) { c0 = min(c0, smem_i[w * 2]); l0 = max(l0, smem_i[w * 2 + 1]); }
                int id = (c0 != INT_MAX) ? c0 : l0;
                if (id < 0) id = 0;
                A.row_id[row] = id;
            }
        }
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
    const int64_t lo = w * K;
    const int64_t hi = (lo + K < N) ? lo + K : N;
    int64_t n = 0;
    while (lo + n < hi && accept[lo + n]) ++n;
    if (accept_len) accept_len[w] = (int32_t)n;
    if (resampled_id) resampled_id[w] = (lo + n < hi) ? row_id[lo + n] : -1;
}

// ---- dense export (tests / debugging): same per-token arithmetic, three sweeps over global memory --------

template <typename T>
__device__ __forceinline__ float load_elt(const T* p, int i)
{
    if constexpr (sizeof(T) == 4) return reinterpret_cast<const float*>(p)[i];
    else return bits_f((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
}

template <typename T>
__global__ __launch_bounds__(256) void dense_kernel(const RowArgs A, float* __restrict__ p_lo,
                                                    float* __restrict__ p_mid, float* __restrict__ p_hi)
{
    constexpr int NW = 4;
    __shared__ double smem[NW * 5];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int V = A.V;
    const T* c = static_cast<const T*>(A.draft) + row * A.stride;

    float m = -INFINITY;
    for (int i = tid; i < V; i += 256) m = fmaxf(m, load_elt(c, i));
    m = block_max<NW>(m, smem, lane, wave);

    double s1[1] = {0.0};
    {
        double acc = 0.0;
        for (int i = tid; i < V; i += 256) acc += (double)exp_shifted(load_elt(c, i), m);
        s1[0] = acc;
    }
    block_sum<NW, 1>(s1, smem, lane, wave);
    const double S = s1[0];

    const FuseRow fr = fuse_row(S, A.a, A.b);
    double q5[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
    {
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0, a4 = 0.0;
        for (int i = tid; i < V; i += 256) {
            float gl, gw;
            fuse_token(exp_shifted(load_elt(c, i), m), fr, gl, gw);
            const double dl = (double)gl, dw = (double)gw;
            a0 += dl; a1 += dw;
            a2 = fma(dl, dl, a2); a3 = fma(dw, dw, a3); a4 = fma(dl, dw, a4);
        }
        q5[0] = a0; q5[1] = a1; q5[2] = a2; q5[3] = a3; q5[4] = a4;
    }
    block_sum<NW, 5>(q5, smem, lane, wave);
    const RowScore rs = finish_score(q5, S, A);

    const float Bc = (float)(A.b / S), Wc = (float)((A.a - A.b) / S), invS = (float)(1.0 / S);
    const float al = (float)rs.alpha_l, au = (float)rs.alpha_u;
    for (int i = tid; i < V; i += 256) {
        const float e = exp_shifted(load_elt(c, i), m);
        float gl, gw;
        fuse_token(e, fr, gl, gw);
        const float pl = Bc * gl;
        const float pu = fmaf(Wc, gw, pl);
        const int64_t o = row * (int64_t)V + i;
        if (p_lo) p_lo[o] = al * pl;
        if (p_mid) p_mid[o] = e * invS;
        if (p_hi) p_hi[o] = au * pu;
    }
}

// ---- dispatch ---------------------------------------------------------------------------------------------

template <typename T, int THREADS, int NVEC>
hipError_t launch_cfg(Mode mode, const RowArgs& a, hipStream_t s)
{
    const dim3 grid((unsigned)a.N), block(THREADS);
    switch (mode) {
    case Mode::Quantify: hipLaunchKernelGGL((row_kernel<T, THREADS, NVEC, true, false>), grid, block, 0, s, a); break;
    case Mode::Verify:   hipLaunchKernelGGL((row_kernel<T, THREADS, NVEC, false, true>), grid, block, 0, s, a); break;
    case Mode::Fused:    hipLaunchKernelGGL((row_kernel<T, THREADS, NVEC, true, true>), grid, block, 0, s, a); break;
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_typed(Mode mode, const RowArgs& a, hipStream_t s)
{
    const int vecs = (a.V + Elt<T>::kPerVec - 1) / Elt<T>::kPerVec;   // 16-byte vectors per row
    if (vecs <= 256 * 1)  return launch_cfg<T, 256, 1>(mode, a, s);
    if (vecs <= 256 * 2)  return launch_cfg<T, 256, 2>(mode, a, s);
    if (vecs <= 256 * 4)  return launch_cfg<T, 256, 4>(mode, a, s);
    if (vecs <= 256 * 8)  return launch_cfg<T, 256, 8>(mode, a, s);
    if (vecs <= 256 * 16) return launch_cfg<T, 256, 16>(mode, a, s);
    if (vecs <= 1024 * 8) return launch_cfg<T, 1024, 8>(mode, a, s);
    return hipErrorInvalidValue;
}

}  // namespace

int max_vocab(int dtype) { return dtype == 0 ? 1024 * 8 * 4 : 1024 * 8 * 8; }

hipError_t launch_rows(Mode mode, int dtype, const RowArgs& args, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    return dtype == 0 ? launch_typed<float>(mode, args, stream) : launch_typed<bf16_t>(mode, args, stream);
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

}  // namespace ciar
