// gfx950 kernels around the streaming kernel: the fp64 pass over flat rows, the window outputs for launches whose
// windows do not lie inside one workgroup, and the arg-max index for tensor-radius calls without drafted ids.
// (Eq. uncertainty_score; Algorithm 1's verification step.)
#include "ciar_device.h"

namespace ciar {
namespace {

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

// Residual draw of the rejected rows (accept bit 0) of launches whose streaming kernel does not draw them itself
// (launches whose tiles do not hold both rows in registers: bf16, the 16-vector fp32 tile, wide radii):
// res_i = max(0, q_i - p_i), inverse CDF in token order; both rows are fetched again, four vectors of each row per
// lane in flight at once.  A row's draw is a chain of dependent steps (statistics, loads, totals, crossing chunk,
// scan), so what matters is how many rows a compute unit has in flight: 256-lane workgroups, several per compute
// unit, unless the launch is so small that most compute units would see no rejected row at all (then 1024 lanes
// work on each row).
// Which workgroup draws which row is settled without a list and without atomic operations (a counter that every
// workgroup of a launch adds to is served one addition after another: a thousand of them cost ~20 us at the end of
// a kernel).  Up to kRankAllRows rows every workgroup reads all the marks, 4096 at a time, ranks the marked rows
// in row order and takes ranks g, g + G, ...: the rows are dealt out evenly whatever their pattern.  Beyond that a
// workgroup takes the marked rows of its own slice of N / G consecutive rows (many rows per slice: even enough).
constexpr int kRankAllRows = 65536;

template <typename T, int THREADS>
__global__ __launch_bounds__(THREADS) void resample_kernel(const RowArgs A, const int K, int32_t* __restrict__ resampled_id)
{
    using E = Elt<T>;
    constexpr int EPV = E::kPerVec;
    constexpr int NW = THREADS / 64;
    constexpr int CHUNK = THREADS * EPV;
    constexpr int MAXCH = 8192 / THREADS;           // chunks of CHUNK tokens a row can have (supported vocabularies)
    constexpr int UB = 4;                           // chunks of each row in flight per lane
    constexpr int SCAN = 4096, MPL = SCAN / THREADS;   // marks read per step of the search, and per lane

    __shared__ double sm_e[NW * MAXCH + NW];
    __shared__ __attribute__((aligned(16))) double sm_q[NW][8][16];   // per wave: [chunk of the group][quad]
    __shared__ int    sm_i[NW * 2];
    __shared__ int    sm_mine[SCAN];                // the rows of a step that this workgroup draws
    __shared__ int    sm_wcount[NW];
    __shared__ int    sm_nmine;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = A.V;
    const int last_vec = (V + EPV - 1) / EPV - 1;
    const int nch = (V + CHUNK - 1) / CHUNK;        // <= MAXCH
    const int64_t N = A.N;
    const int G = (int)gridDim.x, g = (int)blockIdx.x;
    const bool rank_all = N <= kRankAllRows;        // uniform over the grid
    const int64_t slice = (N + G - 1) / G;
    const int64_t lo_row = rank_all ? 0 : (int64_t)g * slice;
    const int64_t hi_row = rank_all ? N : (lo_row + slice < N ? lo_row + slice : N);
    int ranked = 0;                                 // marked rows before this step (rank_all)
    // (a step starts at a multiple of SCAN rows behind lo_row, a lane at a multiple of MPL rows behind that)
    const bool marks_aligned = ((reinterpret_cast<uintptr_t>(A.accept) + (uintptr_t)lo_row) & 15u) == 0;

    for (int64_t s0 = lo_row; s0 < hi_row; s0 += SCAN) {
    // ---- this step's marks: lane t looks at rows s0 + t MPL ... s0 + t MPL + MPL - 1 ------------------------------
    unsigned mask = 0;
    const int64_t r_first = s0 + (int64_t)tid * MPL;
    if (marks_aligned && r_first + MPL <= hi_row) {
        // the lane's MPL accept bytes in one load; they are 0 or 1 (this call's streaming kernel wrote them), so
        // ~w & 0x01010101 has a bit per rejected row, which one multiplication gathers into four adjacent bits
        const uint32_t* w = reinterpret_cast<const uint32_t*>(A.accept + r_first);
        uint32_t words[MPL / 4];
        if constexpr (MPL == 16) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(w);
            words[0] = v.x; words[1] = v.y; words[2] = v.z; words[3] = v.w;
        } else {
#pragma unroll
            for (int i = 0; i < MPL / 4; ++i) words[i] = w[i];
        }
#pragma unroll
        for (int i = 0; i < MPL / 4; ++i)
            mask |= ((((~words[i]) & 0x01010101u) * 0x01020408u) >> 24 & 0xfu) << (4 * i);
    } else {
#pragma unroll
        for (int k = 0; k < MPL; ++k) {
            const int64_t r = r_first + k;
            if (r < hi_row && A.accept[r] == 0) mask |= 1u << k;
        }
    }
    const int mine_cnt = __popc(mask);
    const int incl = (int)wave_scan((double)mine_cnt);             // exact: small integers
    if (lane == 63) sm_wcount[wave] = incl;
    if (tid == 0) sm_nmine = 0;
    __syncthreads();
    int before = ranked + incl - mine_cnt, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        if (w < wave) before += sm_wcount[w];
        total += sm_wcount[w];
    }
    for (int k = 0; k < MPL; ++k) {
        if (mask & (1u << k)) {
            const int row = (int)(s0 + (int64_t)tid * MPL + k);
            if (!rank_all) sm_mine[atomicAdd(&sm_nmine, 1)] = row;          // (any order: each row is drawn on its own)
            else if (before % G == g) sm_mine[atomicAdd(&sm_nmine, 1)] = row;
            ++before;
        }
    }
    ranked += total;
    __syncthreads();
    const int count = sm_nmine;                                    // uniform

    for (int item = 0; item < count; ++item) {
        const int64_t row = sm_mine[item];
        const T* crow = static_cast<const T*>(A.draft) + row * A.stride;
        const T* trow = static_cast<const T*>(A.target) + row * A.stride;
        const RowStats st = A.stats[row];
        const float invSf = (float)(1.0 / st.S), invZf = (float)(1.0 / st.Z);
        const float n = st.n, nt = st.nt;
        const double u_res = (double)A.u_resample[row];

        auto load_vec_nt = [&](const T* base, int j) -> u32x4 {
            const uint32_t off = (uint32_t)min(j * THREADS + tid, last_vec) * 16u;
            return __builtin_nontemporal_load((gvec)((gbytes)base + off));
        };
        auto load_vec = [&](const T* base, int j) -> u32x4 {
            const uint32_t off = (uint32_t)min(j * THREADS + tid, last_vec) * 16u;
            return *(gvec)((gbytes)base + off);
        };
        // residuals of one 16-byte vector of each row; tokens past the end of the row are masked to -inf
        auto residuals = [&](u32x4 cr, u32x4 tr, int j, float (&r)[EPV]) {
            if ((j + 1) * CHUNK > V) {                             // uniform: only the row's last chunk can hold padding
                E::mask_tail(cr, (j * THREADS + tid) * EPV, V);
                E::mask_tail(tr, (j * THREADS + tid) * EPV, V);
            }
            float cv[EPV], tv[EPV];
            E::unpack(cr, cv);
            E::unpack(tr, tv);
            // q - p in fp32: the product e / S is rounded once (6e-8 of p, below the ~1e-7 of p and of q that the fp32
            // exponentials carry anyway) and the FMA forms the difference from the exact product et / Z
#pragma unroll
            for (int k = 0; k < EPV; ++k)
                r[k] = fmaxf(fmaf(exp2_ref(tv[k], nt), invZf, -(exp2_ref(cv[k], n) * invSf)), 0.f);
        };
        // E1: workgroup totals of the residual over each chunk of CHUNK tokens, eight chunks at a time (UB of each row
        // in flight).  The eight lane sums are reduced over the wave together: two DPP steps leave every quad's sums
        // in its lanes, the quad leaders put them into LDS chunk by chunk, lane l takes two of the 16 quad sums of chunk
        // l / 8 and three butterfly steps over its eight lanes finish all eight totals (one DPP reduction of a double
        // over a wave per chunk cost three times as many instructions).
        for (int j0 = 0; j0 < nch; j0 += 8) {
            double ls[8];
#pragma unroll
            for (int half = 0; half < 8 / UB; ++half) {
                u32x4 cb[UB], tb[UB];
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    // (non-temporal: a row is swept once here, and streaming past the caches is what the streaming
                    // kernel's loads do too; workload 5, whose draws are bound by fetching the rows again: 1949 -> 1927 us)
                    cb[u] = load_vec_nt(crow, j0 + half * UB + u);
                    tb[u] = load_vec_nt(trow, j0 + half * UB + u);
                }
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    float sacc = 0.f;
                    if (j0 + half * UB + u < nch) {                // uniform
                        float r[EPV];
                        residuals(cb[u], tb[u], j0 + half * UB + u, r);
#pragma unroll
                        for (int k = 0; k < EPV; ++k) sacc += r[k];
                    }
                    ls[half * UB + u] = (double)sacc;
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                ls[i] = dpp_add<0xB1, 0xf>(ls[i]);                 // lane ^ 1  (quad_perm 1,0,3,2)
                ls[i] = dpp_add<0x4E, 0xf>(ls[i]);                 // lane ^ 2  (quad_perm 2,3,0,1)
            }
            if ((lane & 3) == 0) {
#pragma unroll
                for (int i = 0; i < 8; ++i) sm_q[wave][i][lane >> 2] = ls[i];
            }
            // (the wave reads what its own lanes have written: LDS operations of a wave complete in order)
            const double* pr = &sm_q[wave][lane >> 3][2 * (lane & 7)];
            double a = pr[0] + pr[1];
            a = dpp_add<0xB1, 0xf>(a);
            a = dpp_add<0x4E, 0xf>(a);
            a = dpp_add<0x141, 0xf>(a);                            // the other quad of the eight (row_half_mirror)
            if ((lane & 7) == 0 && j0 + (lane >> 3) < nch) sm_e[wave * MAXCH + j0 + (lane >> 3)] = a;
        }
        __syncthreads();
        // Every wave locates the crossing chunk across its lanes: lane j < nch holds chunk j's total over the
        // waves, an inclusive scan over the lanes gives the running sums in token order, a ballot the first chunk
        // whose running sum exceeds u * R.
        double tot = 0.0;
        if (lane < nch) {
#pragma unroll
            for (int w = 0; w < NW; ++w) tot += sm_e[w * MAXCH + lane];
        }
        const double run = wave_scan(tot);                         // lanes >= nch add nothing
        auto lane_value = [&](double v, int src) {
            return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), src),
                                    __builtin_amdgcn_readlane(__double2loint(v), src));
        };
        const double R = lane_value(run, 63);
        int cand = INT_MAX, lastpos = -1;
        if (R > 0.0) {
            // chunk that holds the crossing of u * R (token order = chunk order, then lane order)
            const double thr = u_res * R;
            const unsigned long long cross = __ballot(lane < nch && run > thr);
            const unsigned long long live = __ballot(lane < nch && tot > 0.0);
            int jstar;
            double before;
            if (cross) {
                jstar = __builtin_amdgcn_readfirstlane(__ffsll((long long)cross) - 1);
                before = jstar > 0 ? lane_value(run, jstar - 1) : 0.0;
            } else {                                               // unreachable for u < 1; keeps the draw valid
                jstar = __builtin_amdgcn_readfirstlane(live ? 63 - __clzll((long long)live) : 0);
                before = R;
            }
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
            if (resampled_id) {
                // the window's draw is its first rejected row's: the rows before this one in its window (inside one
                // workgroup of the streaming kernel, which has written -1 for a window without rejection)
                bool first = true;
                for (int64_t r = row - row % K; first && r < row; ++r) first = A.accept[r] != 0;
                if (first) resampled_id[row / K] = id;
            }
        }
        __syncthreads();                                           // the LDS slots are reused by the next row
    }
    __syncthreads();                                               // sm_mine is rewritten by the next step
    }
}

// ---- flat rows in fp64 ------------------------------------------------------------------------------------------

// The interval sums of the rows that the streaming kernel has marked as flat (RowStats::mode + kSumsFlatPending;
// see needs_flat_pass), redone in fp64 from the logits: e_i = exp(c_i - max c) and the radii with fp64 library
// functions, the InterFuse bounds (App. "Proof of Interval Validity") as they are defined, the five sums about the
// values of the row's first token.  Lane t of a workgroup looks at row 256 b + t; the marked ones are then taken one
// after another by the whole workgroup (they are rare: rows of nearly equal logits).  With `finish` the row's
// quantify outputs are written again as well (launches whose streaming kernel finishes its rows).
template <typename T>
__global__ __launch_bounds__(256) void flatrow_kernel(const RowArgs A, const int finish)
{
    __shared__ int sm_list[256];
    __shared__ int sm_count;
    __shared__ double sm_red[5][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = A.V;
    if (tid == 0) sm_count = 0;
    __syncthreads();
    const int64_t mine = (int64_t)blockIdx.x * 256 + tid;
    if (mine < A.N && A.stats[mine].mode >= kSumsFlatPending) sm_list[atomicAdd(&sm_count, 1)] = tid;
    __syncthreads();
    const int count = sm_count;                                    // uniform
    // (the order of the list varies from run to run, the rows' results do not: each is computed on its own)
    for (int it = 0; it < count; ++it) {
        const int64_t row = (int64_t)blockIdx.x * 256 + sm_list[it];
        const RowStats st = A.stats[row];
        const T* crow = static_cast<const T*>(A.draft) + row_offset(A, row);
        const T* rrow = A.radius ? static_cast<const T*>(A.radius) + row_offset(A, row) : nullptr;
        const double mc = (double)st.mc;
        // the sum of four per-wave sums, in a fixed order
        auto block_sums = [&](double (&v)[5], int n) {
            __syncthreads();                                       // the slots may still be read from the last use
            for (int i = 0; i < n; ++i) {
                const double w = wave_sum(v[i]);
                if (lane == 0) sm_red[i][wave] = w;
            }
            __syncthreads();
            for (int i = 0; i < n; ++i) v[i] = (sm_red[i][0] + sm_red[i][1]) + (sm_red[i][2] + sm_red[i][3]);
        };
        double acc[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
        for (int i = tid; i < V; i += 256) acc[0] += exp((double)load_logit(crow, i) - mc);   // masked token: exp(-inf) = 0
        block_sums(acc, 1);
        const double invS = 1.0 / acc[0];
        auto token = [&](int i, double& pl, double& w) {
            const double x = exp((double)load_logit(crow, i) - mc) * invS;
            double a = A.a, b = A.b;
            if (rrow) {
                const double r = radius_of((double)load_logit(rrow, i), A.kappa, A.rmax);
                a = exp(r); b = exp(-r);
            }
            const double om = 1.0 - x;                             // a flat row: every x is tiny
            pl = b * x / (b + (1.0 - b) * om);
            w = a * x / (1.0 + (a - 1.0) * x) - pl;
        };
        double kl, kw;
        token(0, kl, kw);                                          // every lane forms the same shift
#pragma unroll
        for (int i = 0; i < 5; ++i) acc[i] = 0.0;
        for (int i = tid; i < V; i += 256) {
            double pl, w;
            token(i, pl, w);
            pl -= kl; w -= kw;
            acc[0] += pl; acc[1] += w;
            acc[2] = fma(pl, pl, acc[2]); acc[3] = fma(w, w, acc[3]); acc[4] = fma(pl, w, acc[4]);
        }
        block_sums(acc, 5);
        if (tid == 0) {
            RowStats o = st;
#pragma unroll
            for (int i = 0; i < 5; ++i) o.q[i] = acc[i];
            o.kl = kl; o.kw = kw;
            o.mode = kSumsDirect;
            A.stats[row] = o;
            if (finish) {
                float cx = st.mc, rawx = 0.f;                      // no ids: the arg-max token is reported
                if (A.ids) {
                    int xid = A.ids[ids_index(A, row)];
                    xid = xid < 0 ? 0 : (xid >= V ? V - 1 : xid);
                    cx = load_logit(crow, xid);
                    if (rrow) rawx = load_logit(rrow, xid);
                }
                finish_row(A, row, o, cx, 0.f, rawx, 0.f, true, false);
            }
        }
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
    const T* c = static_cast<const T*>(A.draft) + row_offset(A, row);
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

}  // namespace

hipError_t launch_windows(const uint8_t* accept, const int32_t* row_id, int64_t N, int32_t K,
                          int32_t* accept_len, int32_t* resampled_id, hipStream_t stream);

hipError_t launch_finish(Mode mode, int dtype, const RowArgs& args, const StreamPlan& plan, int32_t K,
                         int32_t* accept_len, int32_t* resampled_id, hipStream_t stream)
{
    if (args.N <= 0 || mode == Mode::Quantify) return hipSuccess;  // the streaming kernel has written every row's outputs
    const bool want_windows = accept_len || resampled_id;
    if (!plan.draws_inline && args.row_id && args.accept) {
        // the rows the streaming kernel has listed; windows inside its workgroups get their draw from here too
        int32_t* const win = want_windows && plan.windows_inline ? resampled_id : nullptr;
        const int64_t cus = compute_units();
        if (args.N >= 4 * cus) {
            // four 256-lane workgroups per compute unit walk over the rejected rows
            if (dtype == 0) hipLaunchKernelGGL((resample_kernel<float, 256>), dim3((unsigned)(4 * cus)), dim3(256), 0, stream, args, K, win);
            else hipLaunchKernelGGL((resample_kernel<bf16_t, 256>), dim3((unsigned)(4 * cus)), dim3(256), 0, stream, args, K, win);
        } else {
            // very few rows (less than one rejected row per compute unit): 1024 lanes on each row
            const unsigned grid = (unsigned)(args.N < cus ? args.N : cus);
            if (dtype == 0) hipLaunchKernelGGL((resample_kernel<float, 1024>), dim3(grid), dim3(1024), 0, stream, args, K, win);
            else hipLaunchKernelGGL((resample_kernel<bf16_t, 1024>), dim3(grid), dim3(1024), 0, stream, args, K, win);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (want_windows && !plan.windows_inline && !plan.windows_counted)
        return launch_windows(args.accept, args.row_id, args.N, K, accept_len, resampled_id, stream);
    return hipSuccess;
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

hipError_t launch_flatrows(int dtype, const RowArgs& args, bool finish_rows, hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)((args.N + 255) / 256)), block(256);
    if (dtype == 0) hipLaunchKernelGGL(flatrow_kernel<float>, grid, block, 0, stream, args, finish_rows ? 1 : 0);
    else hipLaunchKernelGGL(flatrow_kernel<bf16_t>, grid, block, 0, stream, args, finish_rows ? 1 : 0);
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

}  // namespace ciar
