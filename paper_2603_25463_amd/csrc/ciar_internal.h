// Internal interface between the C ABI (ciar_api.cpp) and the gfx950 kernels (ciar_*.hip).
// Not installed; the public contract is include/ciar.h.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace ciar {

// What the streaming kernel leaves per row for the finishing kernel (device workspace).
// Units: e_i = 2^(c_i log2e - n), S = sum e_i; likewise Z with nt for the verifier row.
struct RowStats {
    double S;        // partition sum of the centre row in units of 2^-n
    double Z;        // partition sum of the verifier row in units of 2^-nt
    double q[5];     // InterFuse sums about the shift (kl, kw), units of e: sum (gl - kl), sum (gw - kw),
                     // sum (gl - kl)^2, sum (gw - kw)^2, sum (gl - kl)(gw - kw)
    double kl, kw;   // the shift: gl and gw of the row's first token
    float  n;        // integer-valued reference of the centre row
    float  nt;       // integer-valued reference of the verifier row
    float  mc;       // largest centre logit (the arg-max token's logit)
    float  mode;     // 0 = all five sums; 1 = caps inactive, only q[1], q[3] were accumulated;
                     // 2 = caps inactive and every width above 1/2: q[1], q[3] hold the sums of 1 - width;
                     // 3 = the five sums are of p^l_i and p^u_i - p^l_i themselves (written by the fp64 pass over
                     //     flat rows); + 8 = a flat row that pass has still to visit
};
static_assert(sizeof(RowStats) == 88, "RowStats layout");

// Everything the kernels need, passed by value.  All pointers are device pointers.
struct RowArgs {
    const void*    draft;       // [N, stride] centre logits
    const void*    target;      // [N, stride] verifier logits (verify only)
    const void*    radius;      // [N, stride] raw radius tensor, or null: scalar radius
    const int32_t* ids;         // [N] drafted token (may be null for quantify: arg-max token)
    const float*   u_accept;    // [N]
    const float*   u_resample;  // [N]
    float*   p_lo;  float* p_mid;  float* p_hi;     // [N] or null
    float*   omega; float* sigma;  float* score;    // [N] or null
    uint8_t* flags;                                  // [N] or null
    uint8_t* accept;                                 // [N] or null
    int32_t* row_id;                                 // [N] or null
    RowStats* stats;                                 // [N] workspace
    int32_t* reject_list;                            // [N] workspace ints (the arg-max tokens of a tensor-radius call
                                                     // without drafted ids)
    uint32_t tag;                                    // this launch's tag for the window words (see window_arrive)
    int32_t  finish;                                 // 1 = the streaming kernel also finishes its rows (quantify only)
    // Verification inside the streaming kernel: the accept test, the residual draw of rejected rows from the
    // registers that hold both rows, and the per-row outputs.  A workgroup walks over pieces of `unit` consecutive
    // rows (unit = window: the kernel also writes the window outputs below; unit = 1: a window kernel follows).
    int32_t  unit;
    int32_t  window;                                 // K
    int32_t* accept_len;                             // [ceil(N / K)] or null
    int32_t* resampled_id;                           // [ceil(N / K)] or null
    unsigned long long* win_words;                   // workspace: 16 bytes per row for the words below
    unsigned long long* win_count;                   // win_words or null: windows that span workgroups are written by
                                                     // whichever row of theirs is finished last (window w: the word at
                                                     // byte 16 K w; see window_arrive)
    int32_t  precise_flat;                           // 1 = the streaming kernel marks flat rows for the fp64 pass (see
                                                     // needs_flat_pass)
    int64_t  N;
    int64_t  stride;            // elements between rows
    // Several heads in one launch (quantify only): the N rows are [heads, head_rows], head h starting head_stride
    // elements after head h - 1; head_rows = 0: one head.  ids_period > 0: row r reads ids[r % ids_period] (the
    // heads share one list of drafted tokens).
    int64_t  head_rows;
    int64_t  head_stride;
    int64_t  ids_period;
    int32_t  V;
    int32_t  normalize;
    double   a;                 // e^{+r}   (scalar radius r = min(kappa, rmax))
    double   b;                 // e^{-r}
    double   kappa;             // radius scale: tensor mode r_i = min(kappa Softplus(raw_i), rmax)
    double   rmax;              // radius clamp
    double   tau;
    double   cap_lo;            // 0.99
    double   cap_hi;            // 1.01
    double   capless_xmax;      // rows whose largest probability is below this have inactive caps
    // Scalar radius: (p^u_i - p^l_i) S / ((a - b) e_i) = 1 + x P(x) with P(x) = sum_j wpoly[j] x^j to 2e-8 relative
    // for x = e_i / S <= wpoly_x (negative: no such polynomial for this call)
    float    wpoly[4];
    float    wpoly_x;
};

enum class Mode { Quantify, Verify, Fused };

// Calls whose radius can push every width of a row close to 1 run kernel instances that also accumulate the
// complements of the widths: there the widths crowd against 1, and fp32 widths no longer resolve their own
// spread.  A row's complement sums are used when every 1 - width_i is below 1/2 (the complement is then the
// smaller and the more accurately known of the two).  For that (a - 1) x_i > 1 must hold for the smallest
// probability x_i <= 1 / V, so a = e^r > V is necessary; the instances are chosen from a >= 3 V, because with a
// in between every complement of such a row lies between 1/4 and 1/2, where the two forms are equally accurate.
constexpr double kComplementBelow = 0.5;      // the complement sums are used when every 1 - width is below this
inline bool wide_radius(const RowArgs& a)
{
    const double amax = a.radius ? (a.kappa > 0.0 ? exp(a.rmax) : 1.0) : a.a;
    return amax >= 3.0 * (double)a.V;
}

// Flat rows (largest probability at most 2 / V) whose widths are not small: the widths of such a row can agree to
// 1e-6 and better while their fp32 rounding errors (~1e-7 of each width, uncorrelated as soon as the logits or
// radii differ at all) do not, and U = Omega * Sigma multiplies what those errors leave in Sigma by Omega ~ V * width.
// With uncorrelated errors eps * w per width the score is off by about sqrt(V) * eps * w^2, to be held against its
// absolute tolerance of 1e-7.  A flat row's widths are at most w_cap = 2 a_max / V (a_max = e^r of the largest
// radius the call can produce); calls with sqrt(V) * w_cap^2 above 0.01 -- a hundredth of that tolerance at
// eps = 1e-7 -- mark their flat rows in the streaming kernel and run flatrow_kernel behind it, which redoes those
// rows' interval sums in fp64 from the logits.  The default scalar radius (a = 5.2) stays far below the bound
// for every large vocabulary; tensor-radius calls with the default clamp of 10 are above it.
inline bool needs_flat_pass(const RowArgs& a)
{
    const double amax = a.radius ? (a.kappa > 0.0 ? exp(a.rmax) : 1.0) : a.a;
    double wcap = 2.0 * amax / (double)a.V;
    if (wcap > 1.0) wcap = 1.0;
    return a.V > 64 && wcap * wcap * sqrt((double)a.V) > 0.01;
}

// Largest vocabulary the register-resident streaming kernels cover for an element size.
int max_vocab(int dtype);

// The streaming kernel finishes its own rows: after at most kMaxRowsPerWg rows a workgroup turns what it has parked
// in LDS (statistics, accept decisions, draws) into the rows' outputs, one lane per row, and goes on streaming.
constexpr int kMaxRowsPerWg = 128;

// How a streaming launch over args.N rows would be shaped.
struct StreamPlan {
    unsigned grid;        // workgroups
    int rows_per_wg;      // most rows a workgroup handles
    bool can_finish;      // the kernel finishes its rows (every output of a row but, unless windows_inline, the windows')
    int unit;             // consecutive rows a workgroup takes at a time (launches with a verifier row: 1 or the window)
    bool windows_inline;  // the kernel also writes accept_len / resampled_id (unit == window)
    bool draws_inline;    // the kernel makes the residual draws of rejected rows itself (else resample_kernel follows)
    bool windows_counted; // windows span workgroups, and the kernel still writes accept_len / resampled_id (RowArgs::win_count)
};
StreamPlan plan_stream(Mode mode, int dtype, const RowArgs& args, bool finish_rows = true);

// Streaming pass over the rows: statistics and InterFuse sums into args.stats.  A launch with a verifier row also
// runs the accept test and the residual draws and writes every per-row output (and the window outputs if
// plan_stream says windows_inline); a quantify-only launch writes its per-row outputs if finish_rows is set.
// args needs ids, the uniforms, window and the output pointers accordingly.
// ev_start / ev_stop (both or neither): events the kernel's dispatch records at its start and at its end.
hipError_t launch_stream(Mode mode, int dtype, const RowArgs& args, bool finish_rows, hipStream_t stream,
                         hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// What remains after a streaming pass that has finished its rows: the residual draws of the rejected rows where
// the streaming kernel has only marked them (plan.draws_inline unset), and the window outputs (either may be null)
// for windows of K rows unless the streaming kernel has written them too.
hipError_t launch_finish(Mode mode, int dtype, const RowArgs& args, const StreamPlan& plan, int32_t K,
                         int32_t* accept_len, int32_t* resampled_id, hipStream_t stream);

// The fp64 pass over the rows the streaming kernel has marked as flat (see needs_flat_pass): rewrites their
// RowStats; with finish_rows also their quantify outputs (for launches whose streaming kernel finishes its rows).
hipError_t launch_flatrows(int dtype, const RowArgs& args, bool finish_rows, hipStream_t stream);

// accept_len / resampled_id per window of K rows from the per-row results.
hipError_t launch_windows(const uint8_t* accept, const int32_t* row_id, int64_t N, int32_t K,
                          int32_t* accept_len, int32_t* resampled_id, hipStream_t stream);

// Forward value of the Inter-DRO loss: args.draft = centre logits, args.radius (or null), args.target = cloud
// logits.  terms [7][N]; weights [N] and losses [5] may be null.
hipError_t launch_dro(int dtype, const RowArgs& args, float* terms, double lambda_v, double lambda_p,
                      double lambda_beta, double alpha, float* weights, float* losses, hipStream_t stream);

// Several heads.  Head h of args.draft / args.radius starts h * head_stride elements after head 0;
// args.stats holds [heads][N] RowStats left by one streaming pass per head.
int max_heads();
// Ensemble: token-wise mean of the heads' curves -> the [N] outputs in args.
hipError_t launch_ensemble(int dtype, const RowArgs& args, int heads, int64_t head_stride, hipStream_t stream);
// Ensemble in one sweep (no streaming pass before it, no RowStats): a few heads with a scalar radius whose rows of a
// position fit one workgroup's registers together; every row is read once.  args as for launch_ensemble.
bool ensemble_fused_fits(int dtype, const RowArgs& args, int heads);
hipError_t launch_ensemble_fused(int dtype, const RowArgs& args, int heads, int64_t head_stride, hipStream_t stream);
// Voting: flags[row] = strict majority of head_flags[h * N + row].
hipError_t launch_vote(const uint8_t* head_flags, int heads, int64_t N, uint8_t* flags, hipStream_t stream);

// out[row] = lowest index of the row's largest centre logit.
hipError_t launch_argmax(int dtype, const RowArgs& args, int32_t* out, hipStream_t stream);

// Dense [N, V] export of p_lo, p_mid, p_hi (any may be null).
hipError_t launch_dense(int dtype, const RowArgs& args, float* p_lo, float* p_mid, float* p_hi,
                        hipStream_t stream);

// Plain streaming read of the rows (args.target may be null): the sum of each row's logits.
hipError_t launch_read(int dtype, const RowArgs& args, float* row_sum, hipStream_t stream,
                       hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);

// The Interval Head's two linear maps on the matrix cores: out[n, j] = sum_k hidden[n, k] weight[j, k] + bias[j]
// for the 2V output columns, bf16 operands, fp32 logits; columns [0, V) -> centre, [V, 2V) -> radius.
// The kernel's tile: V must be a multiple of kHeadTileCols and D of kHeadTileDepth (the C ABI checks both).
constexpr int kHeadTileRows = 128, kHeadTileCols = 128, kHeadTileDepth = 64;
struct HeadArgs {
    const uint16_t* hidden;     // [N, D] bf16
    const uint16_t* weight;     // [2V, D] bf16: row j holds the weights of output column j
    const float*    bias;       // [2V] or null
    float*          centre;     // [N, stride] out
    float*          radius;     // [N, stride] out (raw: before Softplus)
    int64_t         N;
    int64_t         stride;     // elements between output rows
    int32_t         D;
    int32_t         V;
    int32_t         row_tiles;  // set by the launcher: tiles of the chosen shape along N
    int32_t         col_tiles;  // and along the 2V output columns
};
hipError_t launch_interhead(const HeadArgs& args, hipStream_t stream, hipEvent_t ev_start = nullptr,
                            hipEvent_t ev_stop = nullptr);

}  // namespace ciar
