// gfx950 kernel of the Interval Head's two linear maps (Sec. 3.2.1, "Interval Head Architecture": the head's
// output dimension is 2 |V|; c_t = Linear_center(h_t), raw radius = Linear_radius(h_t)):
//   out[n, j] = sum_k hidden[n, k] * weight[j, k] + bias[j],   j in [0, 2V)
// bf16 operands, fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16), fp32 logits out: columns
// [0, V) go to the centre rows, [V, 2V) to the raw-radius rows, which the tensor-radius quantifier reads next.
#include "ciar_internal.h"
#include <hip/hip_ext.h>

namespace ciar {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t w32x4 __attribute__((ext_vector_type(4)));

// Workgroup tile 128 x 128 x 64, four waves in a 2 x 2 grid, each wave 64 x 64 = 2 x 2 MFMA blocks of 32 x 32.
constexpr int BM = kHeadTileRows, BN = kHeadTileCols, BK = kHeadTileDepth;
constexpr int PITCH = BK + 8;          // bf16 per LDS row: 144 B, keeps 16-byte alignment and staggers the banks
static_assert(BM == 128 && BN == 128 && BK == 64, "the lane mappings below are written for 128 x 128 x 64");

// Lane layout of v_mfma_f32_32x32x16_bf16: lane l supplies row (A) / column (B) l % 32 with the eight consecutive k
// 8 (l / 32) .. + 7; accumulator register v of lane l is the element (8 (v / 4) + 4 (l / 32) + v % 4, l % 32).
__global__ __launch_bounds__(256) void interhead_gemm_kernel(const HeadArgs A)
{
    __shared__ __attribute__((aligned(16))) uint16_t sA[BM * PITCH];
    __shared__ __attribute__((aligned(16))) uint16_t sB[BN * PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    // consecutive workgroups take the row tiles of one column tile: the weight tile is fetched from HBM once
    const int rt = (int)(blockIdx.x % A.row_tiles), ct = (int)(blockIdx.x / A.row_tiles);
    const int64_t m0 = (int64_t)rt * BM;
    const int n0 = ct * BN;                                        // column of the 2V-wide output

    // staging: a 128 x 64 bf16 tile is 1024 chunks of 16 bytes, four per lane; chunk c = tid + 256 u covers row
    // c / 8, k 8 (c % 8) .. + 7 (eight lanes read 128 consecutive bytes of a row)
    w32x4 ra[4], rb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = tid + 256 * u, r = c >> 3, kc = c & 7;
            int64_t hr = m0 + r;
            if (hr >= A.N) hr = A.N - 1;                           // rows past the end repeat the last one; never stored
            ra[u] = *reinterpret_cast<const w32x4*>(A.hidden + hr * A.D + k0 + kc * 8);
            rb[u] = *reinterpret_cast<const w32x4*>(A.weight + (int64_t)(n0 + r) * A.D + k0 + kc * 8);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = tid + 256 * u, r = c >> 3, kc = c & 7;
            *reinterpret_cast<w32x4*>(&sA[r * PITCH + kc * 8]) = ra[u];
            *reinterpret_cast<w32x4*>(&sB[r * PITCH + kc * 8]) = rb[u];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int lrow = lane & 31, lk = (lane >> 5) * 8;
    fetch(0);
    for (int k0 = 0; k0 < A.D; k0 += BK) {
        stash();
        __syncthreads();
        if (k0 + BK < A.D) fetch(k0 + BK);                         // lands while this tile is multiplied
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[i] = *reinterpret_cast<const bf16x8*>(&sA[(wm * 64 + i * 32 + lrow) * PITCH + kk + lk]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = *reinterpret_cast<const bf16x8*>(&sB[(wn * 64 + j * 32 + lrow) * PITCH + kk + lk]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();                                           // the tile is overwritten next
    }

    // epilogue: bias, then the tile's half of the head (a tile never straddles V: V is a multiple of BN)
    float* out = n0 < A.V ? A.centre : A.radius;
    const int cbase = (n0 < A.V ? n0 : n0 - A.V) + wn * 64 + lrow;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float bj = A.bias ? A.bias[n0 + wn * 64 + j * 32 + lrow] : 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < A.N) out[row * A.stride + cbase + j * 32] = acc[i][j][v] + bj;
            }
    }
}

}  // namespace

hipError_t launch_interhead(const HeadArgs& args, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (args.N <= 0) return hipSuccess;
    const unsigned grid = (unsigned)args.row_tiles * (unsigned)(2 * args.V / BN);
    if (ev_start && ev_stop)
        hipExtLaunchKernelGGL(interhead_gemm_kernel, dim3(grid), dim3(256), 0, stream, ev_start, ev_stop, 0, args);
    else
        hipLaunchKernelGGL(interhead_gemm_kernel, dim3(grid), dim3(256), 0, stream, args);
    return hipGetLastError();
}

}  // namespace ciar
