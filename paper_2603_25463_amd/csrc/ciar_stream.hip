// gfx950 streaming kernel of the CIAR quantify + verify pass (this file), with an overview of the pass.
//
//   stream_kernel   reads every logit row exactly once from HBM.  A workgroup of 256 lanes (512 or 1024 for large
//                   vocabularies or few rows) owns one row at a time and walks over rows blockIdx.x, blockIdx.x +
//                   gridDim.x, ...  The grid is the workgroups that are resident at once (four waves per SIMD;
//                   more, taking their turn, when a workgroup would otherwise get more than kMaxRowsPerWg rows):
//                   while one workgroup waits for its row, the others compute, which keeps the memory system busy
//                   without a second set of row registers.  Loads are interleaved over the workgroup so that every
//                   load instruction of a wave covers 1 KiB of consecutive memory, and non-temporal (every logit is
//                   used once).  Nothing V-wide is ever written back.
//                   What a row leaves behind (its statistics, the accept verdict, the draw of a rejected row) is
//                   parked in LDS, and after its last row the workgroup turns that into the rows' outputs, two
//                   lanes per row in fp64 (finish_batch): caps, Omega, Sigma, U, flag, the interval of the reported
//                   token, the exact accept test, the window outputs.  A call whose rows fit this scheme is this
//                   one launch.
//   resample_kernel (ciar_finish.hip) draws for the rejected rows of launches whose tiles cannot keep both rows in
//                   registers (bf16, the 16-vector fp32 tile, wide radii), re-reading the two rows.
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
//   T  verifier row, loaded into the registers the centre row came in (requested before C where the
//      registers allow, else after it): per-wave maximum, Z_w = sum 2^(t_i log2e - nt_w)   (max-trick)
//   -- barrier: the waves exchange their interval sums and (nt_w, Z_w); thread 0 writes RowStats --
//
// finishing lanes / residual draw, per row (Eq. uncertainty_score; Algorithm 1's threshold and verification steps):
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
#include "ciar_device.h"
#include <hip/hip_ext.h>
#include <type_traits>

namespace ciar {
namespace {

// ---- the streaming kernel ---------------------------------------------------------------------------------

// Waves per SIMD the register allocation aims for: the centre row held as floats plus ~40 working
// registers, capped at 4 waves.  Memory latency is hidden by the other resident workgroups of the compute
// unit rather than by fetching ahead into a second set of registers: measured on this chip, three or
// four resident workgroups beat two with a register prefetch of the next row at every vocabulary size.
// (Tensor-radius mode: the raw radius row sits in registers next to the centre row during the interval pass.)
template <typename T, int THREADS, int NVEC, bool RAD, bool DO_V = false>
constexpr int target_waves()
{
    constexpr int ept = NVEC * Elt<T>::kPerVec;                    // one row as floats
    constexpr int fit = 512 / (ept + (RAD ? NVEC * 4 + 8 : 0) + 40);
    constexpr int lo = (THREADS + 255) / 256;                      // waves per SIMD one workgroup needs
    return fit < lo ? lo : (fit > 4 ? 4 : fit);
}

// The interval sums of a flat row are taken about a shift (kl, kw, kc): sum (gl - kl), sum (gw - kw) and their
// second moments.  A row of nearly equal logits has a spread far below its mean width: about the origin the
// difference of the second moment and the squared mean leaves rounding noise of relative size 1e-8 in Sigma,
// which Omega ~ V multiplies; about a point among the data it loses next to nothing.  "Flat" = the largest
// probability is at most 2 / V.  Elsewhere the spread is at least ~1 / sqrt(V) of the mean and plain sums do; a
// shift would even hurt there, because a token far below it keeps only ulp(k) / 2 of absolute accuracy in gl - k,
// which over a row of small tokens adds up to V * 3e-8 * k.
// Scalar radius: the shift is the token function at the mean of the row's e_i, S / V.  Tensor radius: the values
// of the row's first token.  Every wave forms the shift itself in its own units, a power of two away from the
// others', so the shifts agree bit for bit once they are back in row units and the waves' sums simply add.
struct Shift { float kl, kw, kc; };

// Pass C for one lane: the shifted InterFuse sums over the lane's tokens.  gl - kl and gw - kw come out of the
// FMA that would otherwise have been the multiplication g du, g om: the shift costs no instruction.
// Chunks past the end of a row that does not fill the tile are skipped.
// WIDTH_ONLY = the caps are known to be inactive for this row (alpha_l = alpha_u = 1), so
// delta_i = w_i and only the sums of gw are needed.
// SPLIT = see fuse_parts.
// MASK = the row does not fill the tile: slots past its end contribute nothing (they hold e = 0, which would
// otherwise enter as 0 - k).
//
// Small probabilities (WIDTH_ONLY instances).  The raw width per unit of e,
//   G(x) = (1 - x) / ((1 + (a-1) x)(1 - (1-b) x)),   gw = e G(x),
// is a smooth function of x alone, and almost every token of a large vocabulary has a tiny x.  Where all the
// tokens that one instruction of the wave covers (64 lanes x one 16-byte vector) stay below the bound x_thr the
// host has fitted for this call's radius, G comes from a degree-4 polynomial 1 + x P(x) (relative error <= 2e-8,
// below the rounding of the rational form) instead of three FMAs, a product and a reciprocal: five instruction
// issues instead of ten.  The test costs half an issue per token (a running maximum and one compare per vector).
struct WidthPoly { float d0, d1, d2, d3, ethr; };   // gw = e (1 + e (d0 + e (d1 + e (d2 + e d3)))) for e <= ethr

template <int THREADS, int NVEC, int EPV, bool WIDTH_ONLY, bool SPLIT, bool MASK>
__device__ __forceinline__ void fuse_sums(const float (&e)[NVEC * EPV], const FuseRow& fr_in, const WidthPoly& wp,
                                          const Shift& sh, int V, int tid, double (&q5)[5])
{
    // The caller branches between several instances of this pass.  The row constants go through an empty asm
    // so that each instance has its own: otherwise the optimiser hoists the sub-expressions the instances share
    // (1 + cu e for every token of the lane) above the branch and spills them.
    FuseRow fr = fr_in;
    asm volatile("" : "+v"(fr.cu), "+v"(fr.nih));
    // The sums run in fp64 from the first add (fp64 adds and FMAs issue at the fp32 rate on this chip): one
    // token can hold almost all of a sum.
    double a0[2] = {0.0, 0.0}, a1[2] = {0.0, 0.0}, a2[2] = {0.0, 0.0}, a3[2] = {0.0, 0.0}, a4[2] = {0.0, 0.0};
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        if (j * THREADS * EPV >= V) continue;                      // uniform: the chunk holds no token
        if constexpr (WIDTH_ONLY) {
            // e >= 0: the order of the floats is the order of their bit patterns (integer maxima need no
            // canonicalisation of their operands); a negative bound compares below every e
            int big = __float_as_int(e[j * EPV]);
#pragma unroll
            for (int k = 1; k < EPV; ++k) big = max(big, __float_as_int(e[j * EPV + k]));
            if (__builtin_amdgcn_ballot_w64(big > __float_as_int(wp.ethr)) == 0) {   // uniform over the wave
#pragma unroll
                for (int k = 0; k < EPV; ++k) {
                    const float ek = e[j * EPV + k];
                    const float G = fmaf(fmaf(fmaf(fmaf(wp.d3, ek, wp.d2), ek, wp.d1), ek, wp.d0), ek, 1.0f);
                    float sw = fmaf(ek, G, -sh.kw);
                    if (MASK && (j * THREADS + tid) * EPV + k >= V) sw = 0.f;
                    const double dw = (double)sw;
                    a1[k & 1] += dw;
                    a3[k & 1] = fma(dw, dw, a3[k & 1]);
                }
                __builtin_amdgcn_sched_barrier(0);
                continue;
            }
        }
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float g, du, om;
            fuse_parts<SPLIT>(e[j * EPV + k], fr, g, du, om);
            const bool live = !MASK || (j * THREADS + tid) * EPV + k < V;
            float sw = fmaf(g, om, -sh.kw);
            if (!live) sw = 0.f;
            const double dw = (double)sw;
            a1[k & 1] += dw;
            a3[k & 1] = fma(dw, dw, a3[k & 1]);
            if constexpr (!WIDTH_ONLY) {
                float sl = fmaf(g, du, -sh.kl);
                if (!live) sl = 0.f;
                const double dl = (double)sl;
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

// Pass C for calls with a wide radius (see wide_radius): the five shifted sums and the complements
// ec_i = 1 - width_i over the tokens that exist: q[5] = sum (ec - kc), q[6] = sum (ec - kc)^2, q[7] = the
// lane's largest ec.
template <int THREADS, int NVEC, int EPV>
__device__ __forceinline__ void fuse_sums_wide(const float (&e)[NVEC * EPV], const FuseRow& fr, const Shift& sh,
                                               int V, int tid, double (&q)[8])
{
    double acc[7] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    float big = 0.f;
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        if (j * THREADS * EPV >= V) continue;                      // uniform: the chunk holds no token
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float gl, gw, ec;
            fuse_token_wide(e[j * EPV + k], fr, gl, gw, ec);
            if ((j * THREADS + tid) * EPV + k < V) {
                const double dl = (double)(gl - sh.kl), dw = (double)(gw - sh.kw), dc = (double)(ec - sh.kc);
                acc[0] += dl; acc[1] += dw;
                acc[2] = fma(dl, dl, acc[2]); acc[3] = fma(dw, dw, acc[3]); acc[4] = fma(dl, dw, acc[4]);
                acc[5] += dc; acc[6] = fma(dc, dc, acc[6]);
                big = fmaxf(big, ec);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < 7; ++i) q[i] = acc[i];
    q[7] = (double)big;
}

// Pass C for a handful of tokens (V <= kTinyVocab), in fp64 from the fp32 e_i.  With so few tokens the widths
// are O(1) and Sigma can be an exact zero (two tokens: delta_1 = delta_2 identically, because x_1 + x_2 = 1
// holds for the computed x as well); fp32 token arithmetic leaves ~1e-7 there, fp64 keeps the symmetry.
// Same units as fuse_sums / fuse_sums_rad: gl, gw per token with p^l = Bc gl, p^u - p^l = Wc gw; the shift
// (the values of the row's first token, which lane 0 of wave 0 holds) is returned in kq.
// WIDE: also the complement sums of fuse_sums_wide; first_tok = index of the lane's first token.
template <typename T, int EPV, bool RAD, bool WIDE>
__device__ __forceinline__ void fuse_sums_tiny(const float (&e)[EPV], const u32x4& rad, double S_units, double a,
                                               double b, double kappa, double rmax, int first_tok, int V,
                                               double (&q5)[WIDE ? 8 : 5], double (&kq)[3])
{
    float raw[EPV];
    Elt<T>::unpack(rad, raw);
    const double invS = 1.0 / S_units;
    auto token = [&](float ef, float rawf, double& gl, double& gw, double& ec) {
        const double ed = (double)ef, x = ed * invS;
        double ak = a, bk = b;
        if constexpr (RAD) {
            const double r = radius_of((double)rawf, kappa, rmax);
            ak = exp(r); bk = exp(-r);
        }
        const double om = 1.0 - x, du = 1.0 + (ak - 1.0) * x, dl = bk + (1.0 - bk) * om;   // dl = 1 - (1-b) x
        gl = ed / dl; gw = ed * om / (du * dl);
        if constexpr (RAD) { gl *= bk; gw *= ak - bk; }
        ec = (1.0 - 2.0 * (1.0 - bk) * x * om) / (du * dl);
    };
    // the same reference in every lane: lane 0's first token
    const float e_ref = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(e[0])));
    const float raw_ref = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(raw[0])));
    token(e_ref, raw_ref, kq[0], kq[1], kq[2]);
#pragma unroll
    for (int i = 0; i < (WIDE ? 8 : 5); ++i) q5[i] = 0.0;
#pragma unroll
    for (int k = 0; k < EPV; ++k) {
        if (first_tok + k < V) {
            double gl, gw, ec;
            token(e[k], raw[k], gl, gw, ec);
            gl -= kq[0]; gw -= kq[1];
            q5[0] += gl; q5[1] += gw;
            q5[2] = fma(gl, gl, q5[2]); q5[3] = fma(gw, gw, q5[3]); q5[4] = fma(gl, gw, q5[4]);
            if constexpr (WIDE) {
                q5[7] = fmax(q5[7], ec);
                ec -= kq[2];
                q5[5] += ec; q5[6] = fma(ec, ec, q5[6]);
            }
        }
    }
}

// Pass C in tensor-radius mode: every token has its own a_i, b_i from the raw radius row `rad` (as loaded,
// padding already zeroed); the sums are of p^l_i S and (p^u_i - p^l_i) S themselves, about the shift sh.
// WIDE: also the complement sums of fuse_sums_wide.
// UNIT = the radius scale is 1 (see radius_am1).
template <typename T, int THREADS, int NVEC, bool WIDE, bool UNIT>
__device__ __forceinline__ void fuse_sums_rad(const float (&e)[NVEC * Elt<T>::kPerVec], const u32x4 (&rad)[NVEC],
                                              const FuseRow& fr, const RadiusMode& rm, const Shift& sh, int V,
                                              int tid, double (&q5)[WIDE ? 8 : 5])
{
    const float kappa = rm.kappa, rmax = rm.rmax, am1_max = rm.am1_max;
    constexpr int EPV = Elt<T>::kPerVec;
    double a0[2] = {0.0, 0.0}, a1[2] = {0.0, 0.0}, a2[2] = {0.0, 0.0}, a3[2] = {0.0, 0.0}, a4[2] = {0.0, 0.0};
    double c1 = 0.0, c2 = 0.0;
    float big = 0.f;
#pragma unroll
    for (int j = 0; j < NVEC; ++j) {
        if (j * THREADS * EPV >= V) continue;                      // uniform: the chunk holds no token
        float raw[EPV];
        Elt<T>::unpack(rad[j], raw);
#pragma unroll
        for (int k = 0; k < EPV; ++k) {
            float pl, w;
            const bool live = (j * THREADS + tid) * EPV + k < V;
            if constexpr (WIDE) {
                float ec;
                fuse_token_rad_wide<UNIT>(e[j * EPV + k], raw[k], fr, kappa, rmax, am1_max, pl, w, ec);
                if (live) {
                    const double dc = (double)(ec - sh.kc);
                    c1 += dc; c2 = fma(dc, dc, c2);
                    big = fmaxf(big, ec);
                }
            } else {
                fuse_token_rad<UNIT>(e[j * EPV + k], raw[k], fr, kappa, rmax, am1_max, pl, w);
            }
            const double dl = live ? (double)(pl - sh.kl) : 0.0, dw = live ? (double)(w - sh.kw) : 0.0;
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
    if constexpr (WIDE) { q5[5] = c1; q5[6] = c2; q5[7] = (double)big; }
}

// Whether a second row fits in the registers at four waves per SIMD next to the centre row's floats (fp32 tiles of
// up to 8 vectors per lane) ...
// ... during the interval pass, so that the verifier row can be requested ahead of it (scalar radius: with a radius
// tensor that place is taken by the raw radius row);
template <typename T, int NVEC, bool DO_V, bool RAD, bool WIDE>
constexpr bool second_row_early()
{
    return DO_V && !RAD && !WIDE && (NVEC * Elt<T>::kPerVec + NVEC * 4 + 56) * 4 <= 512;
}
// ... behind it, so that a launch with a verifier row makes the residual draws of its rejected rows inside the
// streaming kernel (scalar or tensor radius: by then the verifier row has taken the raw radius row's place).
template <typename T, int NVEC, bool DO_V, bool RAD, bool WIDE>
constexpr bool draws_in_stream()
{
    return DO_V && !WIDE && (NVEC * Elt<T>::kPerVec + NVEC * 4 + 56) * 4 <= 512;
}

// sm_draw / row_id of a rejected row whose draw is still to be made (by resample_kernel)
constexpr int kDrawPending = -2;

template <typename T, int THREADS, int NVEC, bool DO_Q, bool DO_V, bool RAD, bool WIDE>
__global__ __launch_bounds__(THREADS)
__attribute__((amdgpu_waves_per_eu(target_waves<T, THREADS, NVEC, RAD, DO_V>())))
void stream_kernel(const RowArgs A)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec;
    constexpr int EPT = NVEC * EPV;
    constexpr int NW = THREADS / 64;
    constexpr int CHUNK = THREADS * EPV;            // tokens covered by one load instruction of the workgroup
    // The verifier row is requested before the interval pass where a second row fits in the registers at
    // four waves per SIMD next to the centre row's floats (fp32 tiles of up to 8 vectors per lane; measured
    // 51 -> 48.6 us on the benchmark); elsewhere it would spill, and it is requested after the pass.
    constexpr bool EARLY_T = second_row_early<T, NVEC, DO_V, RAD, WIDE>();
    // Quantify-only launches have no verifier row; under the same condition the next centre row is requested
    // before the interval pass instead.
    constexpr bool EARLY_NEXT = !DO_V && !RAD && !WIDE && (EPT + NVEC * 4 + 56) * 4 <= 512;
    // A rejected row's draw needs both rows.  Where two rows fit, the centre row's exponentials simply stay in their
    // registers next to the verifier row and the draw is made here (KEEP_E).  Elsewhere (bf16 tiles, the 16-vector
    // fp32 tile, wide radii) the two do not fit: such rows are only marked, and resample_kernel
    // draws them behind this kernel (measured with the draw here and the centre row fetched again: the branch
    // alone, never taken, cost the bf16 row loop 11 % -- registers and scheduling -- and workload 3 ran 318 against
    // 285 us per step).
    constexpr bool KEEP_E = draws_in_stream<T, NVEC, DO_V, RAD, WIDE>();
    // Fused launches on bf16 rows with a scalar radius: the two interval sums of a row whose caps are inactive and the
    // verifier row's partition sum are reduced over the wave together (wave_sum3) once the verifier row has been summed.
    // (These instances are bound by their vector instructions: workload 5 1951 -> 1905 us.  The fp32 instances, which
    // wait for memory, measured 1 % slower with it and keep one reduction per sum.)
    constexpr bool BATCH3 = DO_Q && DO_V && !RAD && !WIDE && sizeof(T) == 2;
    constexpr int NQ = WIDE ? 8 : 5;                // interval sums a wave hands over
    constexpr int NT = NVEC * NW;                   // pieces of a row in token order: (vector j, wave w) -> j NW + w

    // Exchange slots.  Two barriers per row order every write against every read: the centre-row
    // slots are written before the first and read between the two, the others are written between the
    // two and read after the second, before the next row's first barrier.
    // (the centre-row slots exist twice and rows alternate between them: a row's write-up and its draw read them
    // after the second barrier, when a wave that runs ahead may already be writing the next row's)
    __shared__ float  sm_ref2[2][NW * 2];           // per wave: max centre logit, n_w
    __shared__ double sm_S2[2][NW];                 // per wave: S_w
    __shared__ float  sm_nt[NW];                    // per wave: nt_w
    __shared__ double sm_Z[NW];                     // per wave: Z_w
    __shared__ double sm_q5[NW * NQ];               // per wave: the interval sums, already in row units
    __shared__ double sm_red[BATCH3 ? NW : 1][48];  // per wave: the slots of wave_sum3
    __shared__ double sm_k[3];                      // the shift the sums are taken about (row units), from wave 0
    __shared__ float  sm_e0;                        // e of the row's first token, in the units of wave 0
    // Finishing inside this kernel: the statistics of the rows this workgroup has streamed since its last
    // finishing step (at most kMaxRowsPerWg of them) and, fetched ahead, what their finishing needs from memory:
    // the reported token's centre logit, raw radius and verifier logit, the row's two uniforms.
    __shared__ RowStats sm_rows[kMaxRowsPerWg];
    __shared__ float    sm_fx[kMaxRowsPerWg][4];    // cx, rawx, tx, u_accept
    __shared__ float    sm_ur[DO_V ? kMaxRowsPerWg : 1];
    __shared__ int      sm_draw[DO_V ? kMaxRowsPerWg : 1];   // -1: the drafted token was accepted; else the row's draw
    __shared__ uint8_t  sm_close[DO_V ? kMaxRowsPerWg : 1];  // the fp32 accept test could not decide the row
    __shared__ double   sm_tab[DO_V ? NT : 1];      // residual mass of each piece of a rejected row
    __shared__ __attribute__((aligned(16))) double sm_quad[KEEP_E && NVEC == 8 ? NW : 1][8][16];   // a draw's quad sums
    __shared__ float    sm_auxf[DO_V ? NW : 1];
    __shared__ int      sm_auxi[DO_V ? NW : 1];

    const int tid = threadIdx.x, lane = tid & 63;
    // (uniform over the wave; bf16 instances keep it in a scalar register, so that nothing indexed by it -- the waves'
    // exchange slots in LDS -- is held in vector registers across the row loop: they have none to spare.  The fp32
    // instances measured 1 % slower that way.)
    const int wave = sizeof(T) == 2 ? __builtin_amdgcn_readfirstlane(tid >> 6) : tid >> 6;
    const int V = A.V;
    RadiusMode rm = {false, 0.f, 0.f, 0.f};
    if constexpr (RAD) rm = radius_mode(A);
    const bool partial = V != NVEC * CHUNK;                        // uniform: the row does not fill the tile
    const int last_vec = (V + EPV - 1) / EPV - 1;
    const int nrows = (int)A.N;
    const int step = (int)gridDim.x;

    // Rows live in global memory (address space 1).  Vector j of this lane: scalar row base + 32-bit
    // byte offset.  A row that fills the tile needs one lane offset for all of its vectors (the
    // distance between vectors is a constant on top of the scalar base).  Otherwise vector indices
    // past the end of the row are clamped to its last vector, so every lane loads valid memory
    // unconditionally; tokens that do not exist are set to -inf afterwards.
    // The loads are non-temporal: every logit is used exactly once, and streaming past the caches measured
    // 10-12 % more bandwidth than ordinary loads on this chip (plain read of 2 GiB: 6.2 -> 6.9 TB/s).
    // The base goes through readfirstlane and the lane index through an empty asm: both are opaque
    // to the optimiser, which otherwise turns the sixteen addresses of a row into sixteen 64-bit
    // induction variables, spills them, and serialises the loads on the reloads.
    // `whole` = false: every lane fetches the row's first vectors only (a few cache lines per wave, results unused).
    // The quantify-only loop requests its next row this way when there is none: a request under a branch made the
    // register allocator spill a third of the centre row there (none when the request is unconditional).
    auto load_row = [&](u32x4 (&buf)[NVEC], const void* rows, int r, bool whole = true) {
        const uint64_t b = (uint64_t)(static_cast<const T*>(rows) + row_offset(A, r));
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
        const gbytes base = (gbytes)(((uint64_t)hi << 32) | lo);
        int t = whole ? tid : 0;
        asm volatile("" : "+v"(t));
        if (partial) {
#pragma unroll
            for (int j = 0; j < NVEC; ++j) {
                const uint32_t off = (uint32_t)min(j * THREADS + t, last_vec) * 16u;
                buf[j] = __builtin_nontemporal_load((gvec)(base + off));
            }
        } else {
            const uint32_t off = (uint32_t)t * 16u;
#pragma unroll
            for (int j = 0; j < NVEC; ++j) buf[j] = __builtin_nontemporal_load((gvec)(base + (uint64_t)j * (THREADS * 16u) + off));
        }
    };
    // Verifier row statistics of one wave from the row as loaded: nt_w and Z_w = sum 2^(t_i log2e - nt_w).
    // Any integer reference serves as long as no term overflows and the large terms stay normal numbers, so the
    // sum is first taken about the reference of the centre row's tokens in the same wave (`guess`: verifier
    // logits follow the device model's), which saves the pass for the maximum; a sum outside [2^-40, 2^100]
    // (a verifier row far from its centre row, or a wave without tokens: sum 0) is redone about the wave's own
    // maximum.
    auto verifier_mask = [&](u32x4 (&tb)[NVEC]) {
        if (partial) {
#pragma unroll
            for (int j = 0; j < NVEC; ++j) E::mask_tail(tb[j], (j * THREADS + tid) * EPV, V);
        }
    };
    // (the lane's share of the sum about the reference nref)
    auto verifier_lane_sum = [&](u32x4 (&tb)[NVEC], float nref) {
        float zacc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NVEC; ++j) {
            float tv[EPV];
            E::unpack(tb[j], tv);
#pragma unroll
            for (int k = 0; k < EPV; ++k) zacc[k & 3] += exp2_ref(tv[k], nref);
            __builtin_amdgcn_sched_barrier(0);
        }
        return (double)((zacc[0] + zacc[1]) + (zacc[2] + zacc[3]));
    };
    // (the sum about the guess was out of range: about the wave's own maximum)
    auto verifier_redo = [&](u32x4 (&tb)[NVEC], float& ntw, double& Zw) {
        if (!(Zw >= 0x1p-40 && Zw <= 0x1p100)) {                   // uniform over the wave; also taken by NaN
            float mt = -INFINITY;
#pragma unroll
            for (int j = 0; j < NVEC; ++j) {
                float tv[EPV];
                E::unpack(tb[j], tv);
#pragma unroll
                for (int k = 0; k < EPV; ++k) mt = fmaxf(mt, tv[k]);
            }
            ntw = ref_of(wave_max(mt));
            Zw = wave_sum(verifier_lane_sum(tb, ntw == -INFINITY ? 0.f : ntw));   // an all-masked wave: every term is 2^-inf = 0
        }
    };
    auto verifier_stats = [&](u32x4 (&tb)[NVEC], float guess, float& ntw, double& Zw) {
        verifier_mask(tb);
        ntw = guess == -INFINITY ? 0.f : guess;
        Zw = wave_sum(verifier_lane_sum(tb, ntw));
        verifier_redo(tb, ntw, Zw);
    };

    // ---- which rows this workgroup takes ---------------------------------------------------------------------
    // Pieces of `unit` consecutive rows: piece blockIdx.x, blockIdx.x + gridDim.x, ...  (unit = 1, or the window
    // length when this kernel also writes the window outputs).  The workgroup's rows are numbered L = 0, 1, 2, ...
    // in the order it streams them; with finishing there are at most `cap` of them (whole pieces; the launcher sizes
    // the grid accordingly), and after the last one one lane per row finishes it from what is parked in LDS.
    const bool finish = (DO_V || A.finish) && (DO_Q || DO_V);      // uniform over the grid
    const int unit = DO_V ? A.unit : 1;
    const int cap = (kMaxRowsPerWg / unit) * unit;
    auto row_of = [&](int L) -> int64_t {
        const int u = L / unit;
        return ((int64_t)blockIdx.x + (int64_t)u * step) * unit + (L - u * unit);
    };
    // What the finishing of rows L0 ... L0 + cap - 1 needs from memory (lane t: row L0 + t), in three steps so that
    // the first row's own loads can go in between: fetch_ids requests the reported tokens, fetch_scalars (which
    // waits for them) their logits and the uniforms, park_scalars (which waits for those) leaves them in LDS.
    struct RowScalars { float cx, rawx, tx, ua, ur; bool live; };
    auto fetch_ids = [&](int L0) {
        const int64_t r = row_of(L0 + tid);
        return (tid < cap && r < nrows && A.ids) ? A.ids[ids_index(A, r)] : 0;
    };
    auto fetch_scalars = [&](int L0, int xid) {
        RowScalars f = {0.f, 0.f, 0.f, 0.f, 0.f, false};
        const int64_t r = row_of(L0 + tid);
        if (tid < cap && r < nrows) {
            f.live = true;
            if (A.ids) {
                xid = xid < 0 ? 0 : (xid >= V ? V - 1 : xid);
                f.cx = load_logit(static_cast<const T*>(A.draft) + row_offset(A, r), xid);
                if constexpr (RAD) f.rawx = load_logit(static_cast<const T*>(A.radius) + row_offset(A, r), xid);
                if constexpr (DO_V) f.tx = load_logit(static_cast<const T*>(A.target) + row_offset(A, r), xid);
            }
            if constexpr (DO_V) { f.ua = A.u_accept[r]; f.ur = A.u_resample[r]; }
        }
        return f;
    };
    auto park_scalars = [&](const RowScalars& f) {
        if (f.live) {
            sm_fx[tid][0] = f.cx; sm_fx[tid][1] = f.rawx; sm_fx[tid][2] = f.tx; sm_fx[tid][3] = f.ua;
            if constexpr (DO_V) sm_ur[tid] = f.ur;
        }
    };
    // Finishing of the rows L0 ... L0 + cnt - 1 from what is parked in LDS, two lanes per row in different waves so that
    // the two halves run side by side: lane i < 128 writes row i's statistics and its quantifier outputs (Eq.
    // uncertainty_score, the threshold of Algorithm 1), lane 128 + i its verification outputs; with unit == window
    // also the outputs of the windows (Algorithm 1: the verified prefix of a drafted window and the token that
    // replaces its first rejection).
    auto finish_batch = [&](int L0, int cnt) {
        static_assert(kMaxRowsPerWg == 128 && THREADS >= 256, "two lanes per parked row");
        __syncthreads();
        // (the lane index through an empty asm: otherwise the row indices below are the ones fetch_scalars formed
        // before the first row, kept in registers or spilled for the whole of the row loop)
        int ft = tid;
        asm volatile("" : "+v"(ft));
        // (likewise the piece length: the divisions by it below otherwise start from what the prologue formed)
        int unit_f = unit;
        asm volatile("" : "+s"(unit_f));
        const int i = ft & 127;                                    // the parked row this lane works on
        const bool mine = ft < 256 && i < cnt;
        const bool qjob = mine && ft < 128, vjob = DO_V && mine && ft >= 128;
        const int64_t r = row_of(L0 + i);
        auto quantify_half = [&]() {
            if (qjob) {
                const RowStats st = sm_rows[i];
                A.stats[r] = st;
                if constexpr (DO_Q) {
                    const float cx = A.ids ? sm_fx[i][0] : st.mc;  // no ids: the arg-max token is reported
                    finish_row(A, r, st, cx, 0.f, sm_fx[i][1], 0.f, true, false);
                }
            }
        };
        // (where the row loop has made the accept test and windows span workgroups, the other half has next to nothing
        // to do ahead of the barrier below and a trip to memory and back behind it -- the window arrivals: there the
        // quantify half runs behind the barrier, next to those, instead of ahead of it, where the other lanes would
        // wait for it; measured on the benchmark: 59.0 -> 57.5 us per step together with the early claim)
        const bool q_late = KEEP_E && A.win_count != nullptr;      // uniform
        if (!q_late) quantify_half();
        if constexpr (DO_V) {
            if (vjob) {
                const RowStats& st = sm_rows[i];
                if constexpr (KEEP_E) {
                    // the row loop has decided in fp32 and drawn; rows it found too close to call are decided here
                    if (sm_close[i] && !reject_exact(sm_fx[i][0], sm_fx[i][2], sm_fx[i][3], st.n, st.nt, st.S, st.Z))
                        sm_draw[i] = -1;                           // accepted after all: the draw does not count
                } else {
                    // the accept test (Algorithm 1, "Cloud verification"); a rejected row's draw is resample_kernel's
                    sm_draw[i] = reject_exact(sm_fx[i][0], sm_fx[i][2], sm_fx[i][3], st.n, st.nt, st.S, st.Z)
                                     ? kDrawPending : -1;
                }
            }
            __syncthreads();                                       // the windows below read their rows' final draws
            if (q_late) quantify_half();
            if (vjob) {
                const int id = sm_draw[i];                         // -1, a draw, or kDrawPending
                if (A.accept) A.accept[r] = (uint8_t)(id == -1);
                if (A.row_id) A.row_id[r] = id;
                // (an opaque copy: the reciprocal that the divisions by K below start from is otherwise the one the
                // workgroup formed for its claim ahead of the first row, kept -- spilled -- through the whole row loop)
                int K = A.window;
                asm volatile("" : "+s"(K));
                if (unit_f == K && !A.win_count && (A.accept_len || A.resampled_id) && i % K == 0) {   // pieces start at multiples of K
                    const int64_t left = nrows - r;
                    const int len = (int)(left < K ? left : K);
                    int m = 0;
                    while (m < len && sm_draw[i + m] == -1) ++m;
                    const uint32_t w = (uint32_t)r / (uint32_t)K;
                    if (A.accept_len) A.accept_len[w] = m;
                    // (a pending draw: resample_kernel writes the window's entry when it has drawn that row)
                    if (A.resampled_id && (m == len || sm_draw[i + m] != kDrawPending))
                        A.resampled_id[w] = m < len ? sm_draw[i + m] : -1;
                }
                if constexpr (KEEP_E) {
                    const int64_t w = (int64_t)((uint32_t)r / (uint32_t)K), lo = w * K;
                    if (A.win_count && (i % unit_f == 0 || r == lo)) {
                        // A window that spans workgroups: the consecutive rows of it that this workgroup holds (one
                        // row where the rows are dealt out singly: measured the fastest for such launches, 58.8 us per
                        // step on workload 2 against 63.2 us with four consecutive rows per workgroup, whose two
                        // arrivals per window cost less than their memory access pattern loses) arrive together in the
                        // window's 64-bit word (window_arrive), from the lane of the first of them, and the arrival
                        // that completes the window writes its outputs.
                        const int len = (int)(nrows - lo < K ? nrows - lo : K);
                        const int piece_end = i - i % unit_f + unit_f;
                        int rows = 0, off = 0, mine_id = -1;
                        for (; i + rows < cnt && i + rows < piece_end && r + rows < lo + len; ++rows) {
                            if (mine_id < 0 && sm_draw[i + rows] >= 0) { mine_id = sm_draw[i + rows]; off = (int)(r + rows - lo); }
                        }
                        int first, draw;
                        if (window_arrive(A.win_count + 2 * lo, A.tag, rows, off, mine_id, len, first, draw)) {
                            if (A.accept_len) A.accept_len[w] = first < 0 ? len : first;
                            if (A.resampled_id) A.resampled_id[w] = first < 0 ? -1 : draw;
                        }
                    }
                }
            }
        }
        __syncthreads();
    };

    // This workgroup's rows: its pieces are whole except possibly the very last piece of the launch.
    int my_rows;
    {
        // (in 32 bits: the entry points take fewer than 2^31 rows, and a 64-bit division is ~150 scalar instructions in
        // a chain -- three of them stood between the start of the kernel and its first request for a row)
        const uint32_t b = blockIdx.x, un = (uint32_t)unit, st = (uint32_t)step;
        const uint32_t pieces = ((uint32_t)nrows + un - 1u) / un;
        const uint32_t mine = b < pieces ? (pieces - b + st - 1u) / st : 0u;
        const bool owns_last = mine > 0u && (pieces - 1u - b) % st == 0u;
        my_rows = (int)(mine * un - (owns_last ? pieces * un - (uint32_t)nrows : 0u));
    }

    // The row index is uniform over the workgroup: keep it in a scalar register.
    // A row's centre logits are loaded and worked on first, its verifier logits second: the centre row
    // carries most of the arithmetic (both of its passes), the verifier row only a short one, so
    // little work is left when the last bytes of the launch arrive.
    // The launcher sizes the grid so that a workgroup has at most `cap` rows: they are finished after the last one,
    // when nothing of a row is held in registers any more.
    constexpr int L0 = 0;
    const int cnt = min(cap, my_rows);                             // uniform
    if (cnt <= 0) return;
    int row = __builtin_amdgcn_readfirstlane((int)row_of(L0));
    int in_piece = 0;                                              // rows of the current piece already taken
    const int piece_jump = __builtin_amdgcn_readfirstlane((step - 1) * unit + 1);   // last row of a piece -> first of the next
    // windows that span workgroups: the words this workgroup's rows will arrive in are looked at first of all (see
    // window_claim), so that the answer is back before the first row is
    unsigned long long* claim_word = nullptr;
    unsigned long long claim_seen = 0;
    if constexpr (KEEP_E) {
        if (A.win_count && tid < cnt) {
            const int64_t r = row_of(L0 + tid);
            const int64_t lo = (int64_t)((uint32_t)r / (uint32_t)A.window * (uint32_t)A.window);
            if (tid % unit == 0 || r == lo) {
                claim_word = A.win_count + 2 * lo;
                claim_seen = __hip_atomic_load(claim_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    int first_id = 0;
    if (finish) first_id = fetch_ids(L0);                          // a small load, issued ahead of the first row's
    u32x4 buf[NVEC];                                               // a row as loaded: centre and verifier row in turn
    load_row(buf, A.draft, row);
    // (the logits of the reported tokens are requested behind the row, once their ids are there, and parked when
    // they arrive: that waits for the row as well, which the first pass needs anyway)
    if (finish) park_scalars(fetch_scalars(L0, first_id));
    if constexpr (KEEP_E) {
        if (claim_word) window_claim(claim_word, A.tag, claim_seen);
    }

    if constexpr (THREADS < 1024) {
        if (cnt > 1) __builtin_amdgcn_s_setprio(3);                // (see "Wave priority by progress" at the end of the loop)
    }
    for (int done = 0;; ++done) {                                  // done = rows of this batch already streamed
        const bool has_next = done + 1 < cnt;                      // uniform
        // (the rows are walked without a division: within a piece the next row, at its end the next piece)
        in_piece = in_piece + 1 == unit ? 0 : in_piece + 1;
        const int next = __builtin_amdgcn_readfirstlane(has_next ? (in_piece == 0 ? row + piece_jump : row + 1) : row);
        float raw0 = 0.f;                                          // raw radius of the row's first token
        if constexpr (RAD && DO_Q) raw0 = load_logit(static_cast<const T*>(A.radius) + row_offset(A, row), 0);

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
            // shows there (measured against the fp64 definition).  Adding the tokens of a 16-byte vector pairwise in
            // fp32 first (fp64 only across vectors: 0.9 instructions less per token) was tried and fails parity: where a
            // cap is active Omega = alpha_u S_u - alpha_l S_l is a small difference of numbers near 1 (0.022 from
            // 1.012 - 0.99 in the failing case), which multiplies the 1e-8 that a dominant token's vector loses by 45.
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
        float (&sm_ref)[NW * 2] = sm_ref2[done & 1];
        double (&sm_S)[NW] = sm_S2[done & 1];
        if (lane == 0) {
            sm_ref[wave * 2] = mcw; sm_ref[wave * 2 + 1] = nw;
            sm_S[wave] = Sw;
            if (DO_Q && wave == 0) sm_e0 = e[0];
        }
        __syncthreads();
        // Combining the waves' results.  With eight waves or more every wave does it across its first lanes (lane
        // l < NW takes wave l; the other lanes of the DPP row repeat wave 0, which changes no maximum, and add
        // nothing); with four a short loop is as quick (measured).
        constexpr bool LANES = NW >= 8;
        const int src = lane < NW ? lane : 0;
        // (by_lanes: across the first lanes of the wave, which must all be active; else in a loop)
        auto combine_S = [&](auto by_lanes, float& mc, float& n, double& S) {
            if constexpr (decltype(by_lanes)::value) {
                const float mc_l = sm_ref[src * 2], n_l = sm_ref[src * 2 + 1];
                mc = row16_max(mc_l); n = row16_max(n_l);
                S = row16_sum(lane < NW && n_l != -INFINITY ? sm_S[src] * pow2_of(n_l - n) : 0.0);
            } else {
                mc = sm_ref[0]; n = sm_ref[1];
#pragma unroll
                for (int w = 1; w < NW; ++w) {
                    mc = fmaxf(mc, sm_ref[w * 2]);
                    n = fmaxf(n, sm_ref[w * 2 + 1]);
                }
                S = 0.0;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float rn = sm_ref[w * 2 + 1];
                    if (rn != -INFINITY) S += sm_S[w] * pow2_of(rn - n);
                }
            }
        };
        float mc, n;
        double S;                                                  // in units of 2^-n
        combine_S(std::integral_constant<bool, LANES>{}, mc, n, S);
        const float Sf = (float)S;                                 // for the accept test (see accept_quick)
        const double fw = nw == -INFINITY ? 0.0 : pow2_of(nw - n);     // this wave's e_i are 1/fw too large

        // ---- C: InterFuse sums in this wave's units, rescaled to row units by lane 0 of the wave ---------
        // Caps: S_l <= b / (1 - (1-b) x_max) and S_u >= a / (1 + (a-1) x_max) for the largest probability
        // x_max of the row, so below the host-computed bound on x_max both caps are inactive and the
        // cheaper width-only pass is exact.  Uniform over the workgroup.
        const double emax = (double)exp2_ref(mc, n);               // the row's largest e_i, in row units
        const bool capless = !A.normalize || (!RAD && emax <= A.capless_xmax * S);
        const bool split = emax > 0.5 * S;                         // some x_i above 1/2: 1 - x needs the two-float 1/S
        const bool flat = emax * (double)V <= 2.0 * S;             // largest probability <= 2 / V (see Shift)
        if constexpr (EARLY_NEXT) {
            __builtin_amdgcn_sched_barrier(0);
            if (has_next) load_row(buf, A.draft, next);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (EARLY_T) {
            // the verifier row goes in flight now, into the registers the centre row came in, and lands
            // during the interval pass
            __builtin_amdgcn_sched_barrier(0);
            load_row(buf, A.target, row);
            __builtin_amdgcn_sched_barrier(0);
        }
        float ntw = -INFINITY;                                     // the reference this wave's Z_w is taken about
        bool lane_sums = false;                                    // uniform: q5[1], q5[3] are still the lanes' own sums
        if constexpr (DO_Q) {
            // x_i = e_i fw / S: hand fuse_row the partition sum expressed in this wave's units
            // (fw is a power of two: the division is a change of exponent)
            const double Su = nw == -INFINITY ? 1.0 : ldexp(S, (int)fminf(n - nw, 1000.f));   // S / fw
            // (the call's a, b and polynomial bound through opaque copies in scalar registers: what is derived from
            // them -- a - 1, 1 - b, the bound as a double -- is then formed here, an instruction each, instead of ahead
            // of the row loop, where it is kept in vector registers, or spilled, for all of it)
            double ra = A.a, rb = A.b;
            float wpx = A.wpoly_x;
            if constexpr (sizeof(T) == 2) asm volatile("" : "+s"(ra), "+s"(rb), "+s"(wpx));   // (fp32 instances: no gain, measured)
            const FuseRow fr = fuse_row(Su, ra, rb);
            double q5[NQ];
            auto shift_of = [&](float eref, const FuseRow& r) {
                Shift k;
                k.kc = 0.f;
                if constexpr (RAD) {
                    if constexpr (WIDE) fuse_token_rad_wide(eref, raw0, r, rm, k.kl, k.kw, k.kc);
                    else fuse_token_rad(eref, raw0, r, rm, k.kl, k.kw);
                } else {
                    if constexpr (WIDE) fuse_token_wide(eref, r, k.kl, k.kw, k.kc);
                    else fuse_token<true>(eref, r, k.kl, k.kw);
                }
                return k;
            };
            // The common shift of a flat row (see Shift), 0 elsewhere.  A wave whose units are too far from the
            // row's (scalar radius) or from wave 0's (tensor radius) to form it takes its sums about 0, and its
            // lane 0 moves them to the common shift afterwards.
            bool near = false;
            Shift sh = {0.f, 0.f, 0.f};
            if (flat) {
                if constexpr (RAD) {
                    const float up = sm_ref[1] - nw;               // e0 is 2^up times larger in this wave's units
                    near = fabsf(up) <= 64.f;                      // uniform over the wave; false for inf and nan
                    if (near) sh = shift_of(ldexpf(sm_e0, (int)up), fr);
                } else {
                    near = fw >= 0x1p-64;                          // uniform over the wave
                    if (near) sh = shift_of((float)(Su / (double)V), fr);
                }
            }
            // the width polynomial of this call's radius in this wave's units (x = e / S)
            WidthPoly wp = {0.f, 0.f, 0.f, 0.f, -1.f};
            if constexpr (!RAD && !WIDE) {
                const float is = -fr.nih, is2 = is * is;
                wp.d0 = A.wpoly[0] * is; wp.d1 = A.wpoly[1] * is2; wp.d2 = A.wpoly[2] * (is2 * is);
                wp.d3 = A.wpoly[3] * (is2 * is2);
                wp.ethr = wpx < 0.f ? -1.f : (float)((double)wpx * Su);
                // uniform over the wave: scalar registers (an FMA reads one of them per issue, so d2 stays a vector)
                auto uniform = [](float v) { return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v))); };
                wp.d0 = uniform(wp.d0); wp.d1 = uniform(wp.d1); wp.d3 = uniform(wp.d3); wp.ethr = uniform(wp.ethr);
            }
            double kq[3] = {(double)sh.kl, (double)sh.kw, (double)sh.kc};   // fp64 copy (the tiny path sets its own)
            bool tiny = false;
            if constexpr (NVEC == 1) tiny = V <= kTinyVocab;       // uniform
            if (tiny) {
                if constexpr (NVEC == 1) {
                    if constexpr (RAD) {
                        __builtin_amdgcn_sched_barrier(0);
                        load_row(buf, A.radius, row);
                        E::zero_tail(buf[0], tid * EPV, V);
                    }
                    // all tokens sit in wave 0, whose lane 0 holds the first one
                    fuse_sums_tiny<T, EPV, RAD, WIDE>(e, buf[0], Su, A.a, A.b, A.kappa, A.rmax,
                                                      tid * EPV, V, q5, kq);
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
                if (rm.unit) fuse_sums_rad<T, THREADS, NVEC, WIDE, true>(e, buf, fr, rm, sh, V, tid, q5);
                else         fuse_sums_rad<T, THREADS, NVEC, WIDE, false>(e, buf, fr, rm, sh, V, tid, q5);
#pragma unroll
                for (int i = 0; i < 5; ++i) q5[i] = wave_sum(q5[i]);
            } else if constexpr (WIDE) {
                fuse_sums_wide<THREADS, NVEC, EPV>(e, fr, sh, V, tid, q5);
#pragma unroll
                for (int i = 0; i < 5; ++i) q5[i] = wave_sum(q5[i]);
            } else if (capless) {
                if (partial)    fuse_sums<THREADS, NVEC, EPV, true, true, true>(e, fr, wp, sh, V, tid, q5);
                else if (split) fuse_sums<THREADS, NVEC, EPV, true, true, false>(e, fr, wp, sh, V, tid, q5);
                else            fuse_sums<THREADS, NVEC, EPV, true, false, false>(e, fr, wp, sh, V, tid, q5);
                if constexpr (BATCH3) {
                    // reduced below, together with the verifier row's sum; until then the quads' sums wait in LDS
                    // (slot addresses from an opaque copy of the lane index: hoisted out of the row loop they are spilled)
                    lane_sums = true;
                    int ol = tid;
                    asm volatile("" : "+v"(ol));
                    wave_sum3_put(q5[1], sm_red[ol >> 6], 0, ol & 63);
                    wave_sum3_put(q5[3], sm_red[ol >> 6], 1, ol & 63);
                } else {
                    q5[1] = wave_sum(q5[1]);
                    q5[3] = wave_sum(q5[3]);
                }
            } else {
                if (partial) fuse_sums<THREADS, NVEC, EPV, false, true, true>(e, fr, wp, sh, V, tid, q5);
                else         fuse_sums<THREADS, NVEC, EPV, false, true, false>(e, fr, wp, sh, V, tid, q5);
#pragma unroll
                for (int i = 0; i < 5; ++i) q5[i] = wave_sum(q5[i]);
            }
            if constexpr (WIDE) {
                q5[5] = wave_sum(q5[5]);
                q5[6] = wave_sum(q5[6]);
                q5[7] = (double)wave_max((float)q5[7]);
            }
            if constexpr (BATCH3) {
                // ---- T (these instances): verifier row statistics, per wave ----------------------------------------
                if constexpr (!EARLY_T) {
                    // no registers to spare next to the interval pass: the verifier row is fetched only now
                    __builtin_amdgcn_sched_barrier(0);
                    load_row(buf, A.target, row);
                }
                verifier_mask(buf);
                ntw = nw == -INFINITY ? 0.f : nw;
                double Zw = verifier_lane_sum(buf, ntw);
                if (lane_sums) {
                    int ol = tid;
                    asm volatile("" : "+v"(ol));
                    wave_sum3_put(Zw, sm_red[ol >> 6], 2, ol & 63);
                    wave_sum3_get(sm_red[ol >> 6], ol & 63, q5[1], q5[3], Zw);
                } else {
                    Zw = wave_sum(Zw);
                }
                verifier_redo(buf, ntw, Zw);
                if (lane == 0) { sm_nt[wave] = ntw; sm_Z[wave] = Zw; }
            }
            if (lane == 0) {
                // to row units (the complements are plain numbers: nothing to rescale)
                double ku = fw;
                const double f2 = fw * fw;
                q5[0] *= fw; q5[1] *= fw; q5[2] *= f2; q5[3] *= f2; q5[4] *= f2;
                if (flat && !near && !tiny) {
                    // Rare: this wave's sums are about 0.  Form the common shift the long way round, in row units
                    // (scalar radius) or in wave 0's (tensor radius), and move the sums to it:  with c = 0 - K and
                    // n tokens,  sum (d - K) = s1 + n c,  sum (d - K)^2 = s2 + 2 c s1 + n c^2,  likewise the cross
                    // moment.
                    double fw0 = 1.0;
                    Shift k0;
                    if constexpr (RAD) {
                        fw0 = pow2_of(sm_ref[1] - n);
                        k0 = shift_of(sm_e0, fuse_row(S / fw0, A.a, A.b));
                    } else {
                        k0 = shift_of((float)(S / (double)V), fuse_row(S, A.a, A.b));
                    }
                    kq[0] = (double)k0.kl * fw0; kq[1] = (double)k0.kw * fw0; kq[2] = (double)k0.kc;
                    ku = 1.0;
                    const double cl = -kq[0], cw = -kq[1], cc = -kq[2];
                    int cnt = 0;                                   // tokens of the row in this wave
                    // (from an opaque copy of the wave's index: the count does not change from row to row, and hoisted
                    // out of the row loop it is kept in registers, or spilled, for all of it)
                    int wv = wave;
                    asm volatile("" : "+v"(wv));
#pragma unroll
                    for (int j = 0; j < NVEC; ++j) cnt += min(max(V - (j * THREADS + wv * 64) * EPV, 0), 64 * EPV);
                    const double nn = (double)cnt;
                    q5[4] += cl * q5[1] + cw * (q5[0] + nn * cl);
                    q5[2] += cl * (2.0 * q5[0] + nn * cl);
                    q5[3] += cw * (2.0 * q5[1] + nn * cw);
                    q5[0] += nn * cl;
                    q5[1] += nn * cw;
                    if constexpr (WIDE) {
                        q5[6] += cc * (2.0 * q5[5] + nn * cc);
                        q5[5] += nn * cc;
                    }
                }
#pragma unroll
                for (int i = 0; i < NQ; ++i) sm_q5[wave * NQ + i] = q5[i];
                if (wave == 0) { sm_k[0] = kq[0] * ku; sm_k[1] = kq[1] * ku; sm_k[2] = kq[2]; }
            }
        }

        // ---- T: verifier row statistics, per wave -----------------------------------------------------------
        if constexpr (DO_V && !BATCH3) {
            double Zw;
            if constexpr (!EARLY_T) {
                // no registers to spare next to the interval pass: the verifier row is fetched only now
                __builtin_amdgcn_sched_barrier(0);
                load_row(buf, A.target, row);
            }
            verifier_stats(buf, nw, ntw, Zw);
            if (lane == 0) { sm_nt[wave] = ntw; sm_Z[wave] = Zw; }
        }
        // The next centre row goes in flight before the barrier and thread 0's bookkeeping -- except where this
        // kernel makes the draws: there both rows stay in the registers until the accept test has been decided (below).
        if constexpr (!EARLY_NEXT && !KEEP_E) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (DO_V) {
                if (has_next) load_row(buf, A.draft, next);
            } else {
                load_row(buf, A.draft, has_next ? next : row, has_next);
            }
        }

        __syncthreads();

        // ---- verification of the drafted token, in every wave alike (Algorithm 1, "Cloud verification") ----------
        // Z and its reference over the waves; the accept test; on a rejection the draw from (q - p)+ by inverse CDF
        // in token order, from the registers: e[] still holds the centre row's exponentials, buf the verifier row.
        // Z and its reference over the waves, exactly (fp64): wanted by the lane that writes the row up and by a draw
        // (by_lanes: across the first lanes of the wave, which must all be active; else in a loop)
        auto combine_Z = [&](auto by_lanes, float& nt, double& Z) {
            nt = -INFINITY;
            Z = 0.0;                                               // in units of 2^-nt
            if constexpr (decltype(by_lanes)::value) {
                const float nt_l = sm_nt[src];
                nt = row16_max(nt_l);
                Z = row16_sum(lane < NW && nt_l != -INFINITY ? sm_Z[src] * pow2_of(nt_l - nt) : 0.0);
            } else {
#pragma unroll
                for (int w = 0; w < NW; ++w) nt = fmaxf(nt, sm_nt[w]);
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float rt = sm_nt[w];
                    if (rt != -INFINITY) Z += sm_Z[w] * pow2_of(rt - nt);
                }
            }
        };
        // (Where resample_kernel makes the draws nothing in this loop depends on the accept test: the lane that
        // finishes the row evaluates it, in fp64.)
        if constexpr (DO_V && KEEP_E) {
            // for the accept test in fp32 a float Z does (every wave evaluates it: kept short)
            float ntq = -INFINITY, Zq = 0.f;
            if constexpr (LANES) {
                const float nt_l = sm_nt[src];
                ntq = row16_max(nt_l);
                Zq = row16_sum_f(lane < NW && nt_l != -INFINITY ? ldexpf((float)sm_Z[src], (int)fmaxf(nt_l - ntq, -200.f)) : 0.f);
            } else {
#pragma unroll
                for (int w = 0; w < NW; ++w) ntq = fmaxf(ntq, sm_nt[w]);
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float rt = sm_nt[w];
                    if (rt != -INFINITY) Zq += ldexpf((float)sm_Z[w], (int)fmaxf(rt - ntq, -200.f));
                }
            }
            const float cx = sm_fx[done][0], tx = sm_fx[done][2], ua = sm_fx[done][3];
            // 1 = accepted, 0 = rejected, -1 = too close to call in fp32: then the draw is made as well, and the
            // lane that finishes the row decides in fp64 whether it counts (about one row in a few thousand)
            const int verdict = accept_quick(cx, tx, ua, n, ntq, Sf, Zq);
            if (tid == 0) sm_close[done] = (uint8_t)(verdict < 0);
            if (verdict > 0) {
                if (tid == 0) sm_draw[done] = -1;
            } else {
                // p_i = e_i pfac, q_i = 2^(t_i log2e - ntw) qfac, res_i = max(0, q_i - p_i) rounded to fp32: every
                // partial sum below is a sum of those floats, so that the totals of the pieces and the running sum
                // inside the piece that holds u R are sums of the same numbers
                // (the lane index goes through an empty asm, so that nothing of this branch is computed ahead of the
                // row loop and kept in registers, or spilled, for all of it)
                int dt = tid;
                asm volatile("" : "+v"(dt));
                const int dlane = dt & 63, dwave = dt >> 6;
                // the row's scalars again, from the exchange slots (nothing of them is kept in registers for this
                // branch; the slots are this row's until the next row's second barrier)
                float dmc, n, nt;
                double S, Z;
                combine_S(std::integral_constant<bool, LANES>{}, dmc, n, S);
                combine_Z(std::integral_constant<bool, LANES>{}, nt, Z);
                const float nw = sm_ref[dwave * 2 + 1], ntw = sm_nt[dwave];
                const double fw = nw == -INFINITY ? 0.0 : pow2_of(nw - n);
                // q - p in fp32, as resample_kernel forms it: the product e / S is rounded once (6e-8 of p, below the ~1e-7
                // of p and of q that the fp32 exponentials carry anyway) and the FMA takes the difference from the exact
                // product of the verifier's exponential and 1 / Z
                const float pfac = (float)(fw / S);
                float ntref = ntw == -INFINITY ? 0.f : ntw;
                // (opaque to the optimiser, like e below: it would otherwise keep the streaming passes' conversions
                // and exponentials of every token alive for this branch, in registers the hot path does not have)
                asm volatile("" : "+v"(ntref));
                const float qfac = (float)((ntw == -INFINITY ? 0.0 : pow2_of(ntw - nt)) / Z);
                auto residuals = [&](int j, float (&r)[EPV]) {
                    float tv[EPV];
                    E::unpack(buf[j], tv);
#pragma unroll
                    for (int k = 0; k < EPV; ++k) {
                        float ek = e[j * EPV + k];
                        asm volatile("" : "+v"(ek));
                        r[k] = fmaxf(fmaf(exp2_ref(tv[k], ntref), qfac, -(ek * pfac)), 0.f);
                    }
                };
                // Piece totals.  Eight vectors per lane: the eight lane sums are reduced over the wave together -- two DPP
                // steps leave every quad's sum in its lanes, the quad leaders put it into LDS vector by vector, then lane l
                // takes two of the 16 quad sums of vector l / 8 and three butterfly steps over its eight lanes finish all
                // eight totals (a DPP reduction of one double over a wave is ~36 instructions: eight of them were a third
                // of a draw).  Fewer vectors: one reduction each.
#pragma unroll
                for (int j = 0; j < NVEC; ++j) {
                    float sj = 0.f;
                    if (j * CHUNK < V) {                           // uniform: the vector holds tokens
                        float r[EPV];
                        residuals(j, r);
#pragma unroll
                        for (int k = 0; k < EPV; ++k) sj += r[k];
                    }
                    if constexpr (NVEC == 8) {
                        double q = (double)sj;
                        q = dpp_add<0xB1, 0xf>(q);                 // lane ^ 1  (quad_perm 1,0,3,2)
                        q = dpp_add<0x4E, 0xf>(q);                 // lane ^ 2  (quad_perm 2,3,0,1)
                        if ((dlane & 3) == 0) sm_quad[dwave][j][dlane >> 2] = q;
                    } else {
                        const double ws = wave_sum((double)sj);
                        if (dlane == 0) sm_tab[j * NW + dwave] = ws;
                    }
                }
                if constexpr (NVEC == 8) {
                    // (the wave reads what its own lanes have written: LDS operations of a wave complete in order)
                    const double* pr = &sm_quad[dwave][dlane >> 3][2 * (dlane & 7)];
                    double t2 = pr[0] + pr[1];
                    t2 = dpp_add<0xB1, 0xf>(t2);
                    t2 = dpp_add<0x4E, 0xf>(t2);
                    t2 = dpp_add<0x141, 0xf>(t2);                  // the other quad of the eight (row_half_mirror)
                    if ((dlane & 7) == 0) sm_tab[(dlane >> 3) * NW + dwave] = t2;
                }
                __syncthreads();
                // every wave locates the piece that holds u R: lane l takes piece l (and l + 64), an inclusive scan
                // over the lanes gives the running sums in token order, a ballot the first one above u R
                constexpr int PER = (NT + 63) / 64;
                double tot[PER], run[PER], carry = 0.0;
                auto lane_value = [&](double v, int from) {
                    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), from),
                                            __builtin_amdgcn_readlane(__double2loint(v), from));
                };
#pragma unroll
                for (int p = 0; p < PER; ++p) {
                    const int idx = p * 64 + dlane;
                    tot[p] = idx < NT ? sm_tab[idx] : 0.0;
                    run[p] = wave_scan(tot[p]) + carry;
                    carry = lane_value(run[p], 63);
                }
                const double R = carry;
                const float ur = sm_ur[done];
                if (R > 0.0) {
                    const double thr = (double)ur * R;
                    int istar = -1;
                    double before = 0.0;
                    double prev_end = 0.0;                         // running sum at the end of the part before
#pragma unroll
                    for (int p = 0; p < PER; ++p) {
                        const unsigned long long cross = __ballot(p * 64 + dlane < NT && run[p] > thr);
                        if (istar < 0 && cross) {
                            const int l = __builtin_amdgcn_readfirstlane(__ffsll((long long)cross) - 1);
                            istar = p * 64 + l;
                            before = l > 0 ? lane_value(run[p], l - 1) : prev_end;
                        }
                        prev_end = lane_value(run[p], 63);
                    }
                    if (istar < 0) {                               // unreachable for u < 1; keeps the draw valid
#pragma unroll
                        for (int p = 0; p < PER; ++p) {
                            const unsigned long long live = __ballot(p * 64 + dlane < NT && tot[p] > 0.0);
                            if (live) istar = p * 64 + __builtin_amdgcn_readfirstlane(63 - __clzll((long long)live));
                        }
                        before = R;
                    }
                    const int wstar = istar % NW, jstar = istar / NW;
                    if (dwave == wstar) {
                        int cand = INT_MAX, lastpos = -1;
#pragma unroll
                        for (int j = 0; j < NVEC; ++j) {
                            if (j == jstar) {                      // uniform; the register arrays keep constant indices
                                float r[EPV];
                                residuals(j, r);
                                float s = 0.f;
#pragma unroll
                                for (int k = 0; k < EPV; ++k) s += r[k];
                                const double incl = wave_scan((double)s);
                                double cum = before + (incl - (double)s);
                                // smallest token of the piece whose inclusive running sum exceeds u R; tokens without
                                // residual mass cannot be drawn; lastpos covers a crossing lost to rounding at its end
                                const int base = (j * THREADS + dt) * EPV;
#pragma unroll
                                for (int k = 0; k < EPV; ++k) {
                                    cum += (double)r[k];
                                    if (r[k] > 0.f) {
                                        lastpos = base + k;
                                        if (cum > thr && cand == INT_MAX) cand = base + k;
                                    }
                                }
                            }
                        }
                        cand = wave_min_i(cand);
                        lastpos = wave_max_i(lastpos);
                        if (dlane == 0) {
                            const int id = cand != INT_MAX ? cand : lastpos;
                            sm_draw[done] = id < 0 ? 0 : id;
                        }
                    }
                } else {
                    // every residual rounded to zero (q == p to working precision): the draw degenerates to the
                    // lowest-index arg-max of q, which is that of the verifier logits; practically never taken
                    float mt = -INFINITY;
#pragma unroll
                    for (int j = 0; j < NVEC; ++j) {
                        float tv[EPV];
                        E::unpack(buf[j], tv);
#pragma unroll
                        for (int k = 0; k < EPV; ++k) mt = fmaxf(mt, tv[k]);
                    }
                    mt = wave_max(mt);
                    if (dlane == 0) sm_auxf[dwave] = mt;
                    __syncthreads();
#pragma unroll
                    for (int w = 0; w < NW; ++w) mt = fmaxf(mt, sm_auxf[w]);
                    int ci = INT_MAX;
#pragma unroll
                    for (int j = 0; j < NVEC; ++j) {
                        float tv[EPV];
                        E::unpack(buf[j], tv);
#pragma unroll
                        for (int k = 0; k < EPV; ++k) {
                            const int tok = (j * THREADS + dt) * EPV + k;
                            if (tv[k] == mt && tok < V) ci = min(ci, tok);
                        }
                    }
                    ci = wave_min_i(ci);
                    if (dlane == 0) sm_auxi[dwave] = ci;
                    __syncthreads();
                    if (dt == 0) {
                        int c0 = sm_auxi[0];
#pragma unroll
                        for (int w = 1; w < NW; ++w) c0 = min(c0, sm_auxi[w]);
                        sm_draw[done] = c0 == INT_MAX ? 0 : c0;
                    }
                }
            }
            // both rows are spent: the next centre row goes in flight
            __builtin_amdgcn_sched_barrier(0);
            if (has_next) load_row(buf, A.draft, next);
        }

        // ---- wave 0 leaves the row's ten numbers for the finishing -------------------------------------------------
        // Sixteen waves: their results are combined across the first lanes as above; fewer: by lane 0 in a loop
        // (as quick, measured).  Handing this job from wave to wave in turn measured slower.
        if (wave == 0 && (NW >= 16 || lane == 0)) {
            float mc, n, nt = -INFINITY;
            double S, Z = 0.0;
            combine_S(std::integral_constant<bool, (NW >= 16)>{}, mc, n, S);
            if constexpr (DO_V) combine_Z(std::integral_constant<bool, (NW >= 16)>{}, nt, Z);
            double t[NQ];
#pragma unroll
            for (int i = 0; i < NQ; ++i) t[i] = 0.0;
            double K[3] = {0.0, 0.0, 0.0};
            if constexpr (DO_Q) { K[0] = sm_k[0]; K[1] = sm_k[1]; K[2] = sm_k[2]; }
            // the waves' interval sums are about one common shift (wave 0 left it in row units): they simply add
            if constexpr (DO_Q) {
                if constexpr (NW >= 16) {
#pragma unroll
                    for (int i = 0; i < NQ; ++i) {
                        const double mine = lane < NW ? sm_q5[src * NQ + i] : 0.0;
                        t[i] = i == 7 ? (double)row16_max((float)mine) : row16_sum(mine);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < NQ; ++i) {
#pragma unroll
                        for (int w = 0; w < NW; ++w)
                            t[i] = i == 7 ? fmax(t[i], sm_q5[w * NQ + i]) : t[i] + sm_q5[w * NQ + i];
                    }
                }
            }
            if (lane == 0) {
                RowStats stv;
                RowStats* const st = &stv;
                st->S = S; st->Z = Z; st->n = n; st->nt = nt; st->mc = mc;
                float mode = (capless && !WIDE) ? kSumsWidthOnly : kSumsFull;
                if constexpr (WIDE && DO_Q) {
                    // every width above 1/2 and both caps inactive: the finishing reads the complement sums
                    if (t[7] < kComplementBelow) {
                        const RowScore rs = finish_score(t, S, kSumsFull, A, K[0], K[1]);
                        if (rs.alpha_l == 1.0 && rs.alpha_u == 1.0) {
                            t[1] = t[5]; t[3] = t[6]; K[1] = K[2];
                            mode = kSumsComplement;
                        }
                    }
                }
                // a flat row of a call whose widths are not small: the fp64 pass behind this kernel redoes its sums
                if (DO_Q && A.precise_flat && flat && V > kTinyVocab) mode += kSumsFlatPending;
                st->kl = K[0]; st->kw = K[1];
                st->mode = mode;
#pragma unroll
                for (int i = 0; i < 5; ++i) st->q[i] = t[i];
                // with finishing the statistics stay in LDS until the batch is finished
                if (finish) sm_rows[done] = stv;
                else A.stats[row] = stv;
            }
        }

        if (!has_next) break;
        row = next;
        // Wave priority by progress (set here for the next row; the first row runs at priority 3): the workgroups of a compute unit are served oldest first, so the one that was
        // dispatched first runs at full speed and the others on what it leaves (a timeline of the benchmark launch: the
        // first workgroup of every compute unit took 7.5 us per row and ended at 39 us, the second 12 us per row and ended
        // at 49 us, alone on its compute unit for the last 10 us).  A workgroup therefore runs the first quarter of its
        // rows at priority 3, the second at 2, ...: whoever is behind is served first, and the workgroups of a compute
        // unit end together (benchmark 55.6 -> 52.8 us per step, workload 4 347 -> 328 us, workload 3 276 -> 257 us).
        // Not where a compute unit holds one workgroup only (1024 lanes), and not for a single row.
        if constexpr (THREADS < 1024) {
            if (cnt > 1) {
                // (uniform; floor(4 done / cnt) without a division: compares and shifts on scalar registers)
                if ((done + 1) < ((cnt + 3) >> 2)) __builtin_amdgcn_s_setprio(3);
                else if ((done + 1) < ((cnt + 1) >> 1)) __builtin_amdgcn_s_setprio(2);
                else if ((done + 1) < ((3 * cnt + 3) >> 2)) __builtin_amdgcn_s_setprio(1);
                else __builtin_amdgcn_s_setprio(0);
            }
        }
    }
    if (finish) finish_batch(L0, cnt);
}

// ---- dispatch ---------------------------------------------------------------------------------------------

// A launch request: with `launch` unset the dispatch below only reports the grid it would use.
struct StreamLaunch {
    bool launch;
    bool finish_rows;      // the caller wants the kernel to finish its rows (launches with a verifier row always do)
    hipStream_t stream;
    StreamPlan plan;       // out
    hipEvent_t ev_start, ev_stop;   // both or neither: recorded by the dispatch at the kernel's start and end
};

template <typename T, int THREADS, int NVEC, bool DO_Q, bool DO_V, bool RAD, bool WIDE = false>
hipError_t launch_stream_kernel(const RowArgs& a, StreamLaunch& L)
{
    // One wave of resident workgroups, each walking over its pieces of rows with stride gridDim.x.  The register
    // budget the kernel was compiled for fixes how many fit: target_waves() waves per SIMD, and a
    // workgroup puts THREADS / 256 waves on each of the four SIMDs of a compute unit (a 128-lane one: one
    // wave on two of them).
    constexpr int per_cu = target_waves<T, THREADS, NVEC, RAD, DO_V>() * 256 / THREADS;
    const int64_t resident = (int64_t)per_cu * compute_units();
    const int64_t N = a.N;
    // (at most kMaxRowsPerWg rows per workgroup: beyond that many rows per resident workgroup the grid grows instead)
    auto grid_for = [&](int64_t pieces, int64_t per_wg) {
        const int64_t g = pieces < resident ? pieces : resident, need = (pieces + per_wg - 1) / per_wg;
        return g > need ? g : need;
    };
    const int64_t grid1 = grid_for(N, kMaxRowsPerWg), max1 = (N + grid1 - 1) / grid1;
    StreamPlan& p = L.plan;
    p.unit = 1;
    p.grid = (unsigned)grid1;
    p.rows_per_wg = (int)max1;
    p.windows_inline = false;
    if (DO_V && (a.accept_len || a.resampled_id) && a.window >= 1 && a.window <= kMaxRowsPerWg) {
        // Whole windows per workgroup, so that the kernel writes the window outputs as well, unless that would leave
        // the busiest workgroup with noticeably more rows than a row-by-row split (few windows on many compute units)
        const int64_t K = a.window, units = (N + K - 1) / K;
        const int64_t gridk = grid_for(units, kMaxRowsPerWg / K), maxk = (units + gridk - 1) / gridk * K;
        if (maxk <= max1 + max1 / 8) {
            p.unit = (int)K;
            p.grid = (unsigned)gridk;
            p.rows_per_wg = (int)maxk;
            p.windows_inline = true;
        }
    }
    p.can_finish = DO_V || L.finish_rows;
    p.draws_inline = draws_in_stream<T, NVEC, DO_V, RAD, WIDE>();
    // Windows that span workgroups: where this kernel knows every row's draw it can still write the window outputs,
    // from the lane that finishes a window's last row (one 64-bit word per window in the workspace, see window_arrive).
    p.windows_counted = p.draws_inline && a.win_words && (a.accept_len || a.resampled_id) && !p.windows_inline && a.window >= 2 &&
                        a.window <= kMaxCountedWindow;

    if (!L.launch) return hipSuccess;
    RowArgs b = a;
    b.finish = p.can_finish ? 1 : 0;
    b.unit = p.unit;
    b.win_count = p.windows_counted ? a.win_words : nullptr;
    if (L.ev_start && L.ev_stop)
        hipExtLaunchKernelGGL((stream_kernel<T, THREADS, NVEC, DO_Q, DO_V, RAD, WIDE>), dim3(p.grid), dim3(THREADS),
                              0, L.stream, L.ev_start, L.ev_stop, 0, b);
    else
        hipLaunchKernelGGL((stream_kernel<T, THREADS, NVEC, DO_Q, DO_V, RAD, WIDE>), dim3(p.grid), dim3(THREADS), 0,
                           L.stream, b);
    return hipGetLastError();
}

template <typename T, int THREADS, int NVEC>
hipError_t launch_stream_cfg(Mode mode, const RowArgs& a, StreamLaunch& s)
{
    const bool rad = a.radius != nullptr;
    if (mode != Mode::Verify && wide_radius(a)) {
        // radii at which the widths crowd against 1: the variants that also accumulate their complements
        if (mode == Mode::Quantify)
            return rad ? launch_stream_kernel<T, THREADS, NVEC, true, false, true, true>(a, s)
                       : launch_stream_kernel<T, THREADS, NVEC, true, false, false, true>(a, s);
        return rad ? launch_stream_kernel<T, THREADS, NVEC, true, true, true, true>(a, s)
                   : launch_stream_kernel<T, THREADS, NVEC, true, true, false, true>(a, s);
    }
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
hipError_t launch_stream_typed(Mode mode, const RowArgs& a, StreamLaunch& s)
{
    const int vecs = (a.V + Elt<T>::kPerVec - 1) / Elt<T>::kPerVec;   // 16-byte vectors per row
    if (vecs <= 256 * 1)  return launch_stream_cfg<T, 256, 1>(mode, a, s);
    if (vecs <= 256 * 2)  return launch_stream_cfg<T, 256, 2>(mode, a, s);
    if (vecs <= 256 * 4)  return launch_stream_cfg<T, 256, 4>(mode, a, s);
    if (vecs <= 256 * 8)  return launch_stream_cfg<T, 256, 8>(mode, a, s);
    if (vecs <= 256 * 16) {
        // Few rows: eight waves on a row keep the last rows of the launch short and the grid even; with many
        // rows the four-wave tile has less exchange overhead (measured).  For bf16 the four-wave tile would
        // hold 128 floats per lane and spill: eight waves always.  The same goes for launches with a verifier
        // row, which keep both rows in the registers until the accept test is decided.
        if constexpr (sizeof(T) == 2) {
            return launch_stream_cfg<T, 512, 8>(mode, a, s);
        } else {
            if (mode != Mode::Quantify || a.N < 12 * (int64_t)compute_units()) return launch_stream_cfg<T, 512, 8>(mode, a, s);
            return launch_stream_cfg<T, 256, 16>(mode, a, s);
        }
    }
    if (vecs <= 1024 * 8) return launch_stream_cfg<T, 1024, 8>(mode, a, s);
    return hipErrorInvalidValue;
}

}  // namespace

int max_vocab(int dtype) { return dtype == 0 ? 1024 * 8 * 4 : 1024 * 8 * 8; }

StreamPlan plan_stream(Mode mode, int dtype, const RowArgs& args, bool finish_rows)
{
    StreamLaunch L{false, finish_rows, nullptr, {0u, 0, false, 1, false, false, false}, nullptr, nullptr};
    if (args.N > 0) {
        if (dtype == 0) (void)launch_stream_typed<float>(mode, args, L);
        else (void)launch_stream_typed<bf16_t>(mode, args, L);
    }
    return L.plan;
}

hipError_t launch_stream(Mode mode, int dtype, const RowArgs& args, bool finish_rows, hipStream_t stream,
                         hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (args.N <= 0) return hipSuccess;
    StreamLaunch L{true, finish_rows, stream, {0u, 0, false, 1, false, false, false}, ev_start, ev_stop};
    return dtype == 0 ? launch_stream_typed<float>(mode, args, L)
                      : launch_stream_typed<bf16_t>(mode, args, L);
}

}  // namespace ciar
