// gfx950 kernels that are not steps of the method: the dense [N, V] export of the interval curves (tests,
// debugging) and the plain streaming read that serves as the bandwidth ceiling in benchmarks.
#include "ciar_device.h"
#include <hip/hip_ext.h>

namespace ciar {
namespace {

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
    const RadiusMode rm = radius_mode(A);
    // gl, gw of one token: p^l = Bc gl, p^u - p^l = Wc gw (tensor-radius mode: Bc = Wc = 1 / S)
    auto token = [&](int i, float& e, float& gl, float& gw) {
        e = exp2_ref(load_logit(c, i), n);
        if (rad) fuse_token_rad(e, load_logit(rad, i), fr, rm, gl, gw);
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
    const RowScore rs = finish_score(q5, S, kSumsFull, A, 0.0, 0.0);

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
        for (int j = 0; j < UB; ++j) cb[j] = __builtin_nontemporal_load(&c[min(base + j * 256 + tid, nvec - 1)]);
        if (two) {
#pragma unroll
            for (int j = 0; j < UB; ++j) tb[j] = __builtin_nontemporal_load(&t[min(base + j * 256 + tid, nvec - 1)]);
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

}  // namespace

hipError_t launch_dense(int dtype, const RowArgs& args, float* p_lo, float* p_mid, float* p_hi,
                        hipStream_t stream)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)args.N), block(256);
    if (dtype == 0) hipLaunchKernelGGL(dense_kernel<float>, grid, block, 0, stream, args, p_lo, p_mid, p_hi);
    else hipLaunchKernelGGL(dense_kernel<bf16_t>, grid, block, 0, stream, args, p_lo, p_mid, p_hi);
    return hipGetLastError();
}

hipError_t launch_read(int dtype, const RowArgs& args, float* row_sum, hipStream_t stream, hipEvent_t ev_start,
                       hipEvent_t ev_stop)
{
    if (args.N <= 0) return hipSuccess;
    const dim3 grid((unsigned)args.N), block(256);
    if (ev_start && ev_stop) {
        // the dispatch records the two events at the kernel's start and end
        if (dtype == 0) hipExtLaunchKernelGGL(read_kernel<float>, grid, block, 0, stream, ev_start, ev_stop, 0, args, row_sum);
        else hipExtLaunchKernelGGL(read_kernel<bf16_t>, grid, block, 0, stream, ev_start, ev_stop, 0, args, row_sum);
    } else {
        if (dtype == 0) hipLaunchKernelGGL(read_kernel<float>, grid, block, 0, stream, args, row_sum);
        else hipLaunchKernelGGL(read_kernel<bf16_t>, grid, block, 0, stream, args, row_sum);
    }
    return hipGetLastError();
}

}  // namespace ciar
