// gfx950 kernel of the Interval Head's two linear maps (Sec. 3.2.1, "Interval Head Architecture": the head's
// output dimension is 2 |V|; c_t = Linear_center(h_t), raw radius = Linear_radius(h_t)):
//   out[n, j] = sum_k hidden[n, k] * weight[j, k] + bias[j],   j in [0, 2V)
// bf16 operands, fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16), fp32 logits out: columns
// [0, V) go to the centre rows, [V, 2V) to the raw-radius rows, which the tensor-radius quantifier reads next.
#include <mutex>
#include "ciar_internal.h"
#include <hip/hip_ext.h>

namespace ciar {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Workgroup tile (64 MB) x (64 NB) x 64 with four waves in a 2 x 2 grid, each wave (32 MB) x (32 NB) = MB x NB MFMA
// blocks of 32 x 32.  MB = NB = 4 (256 x 256, a wave 128 x 128) is the shape for real vocabularies: a wave then
// reads 8 operand vectors from LDS for 16 matrix instructions, half the LDS traffic per instruction of the
// 128 x 128 tile (MB = NB = 2), which serves vocabularies that are not a multiple of 256 and very small batches.
//
// Operand tiles go from memory straight into LDS (global_load_lds_dwordx4: no staging registers, and a request
// has a whole tile's multiplication to arrive in).  One such instruction writes the 64 lanes'
// 16-byte chunks to 1 KiB of consecutive LDS, i.e. eight tile rows of 64 bf16 without padding, so the chunks of a
// row are stored in swizzled order instead: chunk q of row r sits at position q ^ ((r / 2) % 8).  The lanes choose which
// chunk of their row they request accordingly (the eight lanes of a row still cover its 128 bytes), and the 32
// rows that one operand read touches at the same k are spread over the banks: a row is 32 banks wide, so the
// even rows share one half of the 64 banks and the odd rows the other, and any 16 consecutive rows (eight of
// each kind, with eight different positions) cover every bank once.
constexpr int BK = kHeadTileDepth;
constexpr int ROWB = BK * 2;            // bytes of a tile row in LDS
static_assert(BK == 64, "a tile row is eight 16-byte chunks");
using gptr = const __attribute__((address_space(1))) void*;
using lptr = __attribute__((address_space(3))) void*;

// Lane layout of v_mfma_f32_32x32x16_bf16: lane l supplies row (A) / column (B) l % 32 with the eight consecutive k
// 8 (l / 32) .. + 7; accumulator register v of lane l is the element (8 (v / 4) + 4 (l / 32) + v % 4, l % 32).
template <int MB, int NB>
__global__ __launch_bounds__(256) void interhead_gemm_kernel(const HeadArgs A)
{
    constexpr int BM = 64 * MB, BN = 64 * NB;
    constexpr int CA = BM / 32, CB = BN / 32;                      // load instructions per wave and tile (8 rows each)
    constexpr int BUF = (BM + BN) * ROWB;                          // bytes of one buffer: the A tile, then the B tile
    extern __shared__ __attribute__((aligned(1024))) char lds[];   // two buffers

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    // Workgroups are handed to the eight XCDs in turn (workgroup b runs on XCD b % 8), and every XCD has an L2 of its
    // own.  So the tiles are dealt by XCD: XCD x takes the column tiles x, x + 8, ..., and its consecutive
    // workgroups walk the row tiles of one column tile.  The workgroups that are resident on an XCD together then
    // share their weight tile (and the few row tiles of hidden states) in that L2.
    int rt, ct;
    if (A.col_tiles % 8 == 0) {
        const int x = (int)(blockIdx.x & 7), local = (int)(blockIdx.x >> 3);
        rt = local % A.row_tiles;
        ct = (local / A.row_tiles) * 8 + x;
    } else {
        rt = (int)(blockIdx.x % A.row_tiles);
        ct = (int)(blockIdx.x / A.row_tiles);
    }
    const int64_t m0 = (int64_t)rt * BM;
    const int n0 = ct * BN;                                        // column of the 2V-wide output

    // Requests: instruction u of wave w covers the tile rows 8 (w + 4 u) .. + 7; lane l asks for row + l / 8 and,
    // of that row, the chunk that belongs at position l % 8.  Addresses: a uniform base per tile plus one 32-bit
    // byte offset per instruction (rows past the end of the batch repeat the last row; they are never stored).
    uint32_t oa[CA], ob[CB];
    const int rl = lane >> 3, chunk = (lane & 7) ^ ((4 * (wave & 1)) | (rl >> 1));   // row = 8 (w + 4 u) + rl: (row / 2) % 8
    const int64_t last = A.N - 1 - m0;                             // >= 0: the tile starts inside the batch
#pragma unroll
    for (int u = 0; u < CA; ++u) {
        const int row = 8 * (wave + 4 * u) + rl;
        oa[u] = (uint32_t)(row <= last ? row : (int)last) * (uint32_t)A.D * 2u + (uint32_t)chunk * 16u;
    }
#pragma unroll
    for (int u = 0; u < CB; ++u) ob[u] = (uint32_t)(8 * (wave + 4 * u) + rl) * (uint32_t)A.D * 2u + (uint32_t)chunk * 16u;
    const char* const baseA = reinterpret_cast<const char*>(A.hidden + m0 * A.D);
    const char* const baseB = reinterpret_cast<const char*>(A.weight + (int64_t)n0 * A.D);
    auto request = [&](int k0, int buf) {
        char* const dA = lds + buf * BUF + wave * 8 * ROWB;
        char* const dB = dA + BM * ROWB;
#pragma unroll
        for (int u = 0; u < CA; ++u)
            __builtin_amdgcn_global_load_lds((gptr)(baseA + k0 * 2 + oa[u]), (lptr)(dA + u * 32 * ROWB), 16, 0, 0);
#pragma unroll
        for (int u = 0; u < CB; ++u)
            __builtin_amdgcn_global_load_lds((gptr)(baseB + k0 * 2 + ob[u]), (lptr)(dB + u * 32 * ROWB), 16, 0, 0);
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Operand reads: lane l reads row l % 32 of each 32-row block; its chunk in slice sl (k 16 sl .. + 15) is
    // 2 sl + l / 32, stored at position (2 sl) ^ sw with sw = (l / 32) ^ ((row / 2) % 8).
    const int lrow = lane & 31, sw = (lane >> 5) ^ ((lrow >> 1) & 7);
    const int offA = (wm * 32 * MB + lrow) * ROWB, offB = BM * ROWB + (wn * 32 * NB + lrow) * ROWB;

    // Pipeline over the k tiles, one barrier per tile.  A tile is multiplied in four 16-deep slices; the operands
    // of a slice are read from LDS during the matrix instructions of the slice before (two register sets), early in
    // it, so that a slice never starts by waiting for LDS.  The barrier stands after the third slice: by then every
    // wave holds its last operands of the current tile in registers, so behind the barrier the tile's buffer is
    // free and the tile after the next is requested into it at once, a whole tile's multiplication ahead of its
    // use; the fourth slice already reads the first operands of the next tile, whose arrival the barrier has
    // awaited (own requests, then the other waves).  Past the last tile the requests repeat it, so no branch
    // splits the loop body; the barrier before the epilogue awaits the last of them.
    static_assert(MB == NB && BK == 64, "the slice pattern below is written for square wave tiles, four slices");
    const int klast = A.D - BK;
    bf16x8 a[2][MB], b[2][NB];
    auto operands = [&](const char* tile, int sl, int set) {
        const int pos = ((2 * sl) ^ sw) * 16;
#pragma unroll
        for (int i = 0; i < MB; ++i) a[set][i] = *reinterpret_cast<const bf16x8*>(tile + offA + i * 32 * ROWB + pos);
#pragma unroll
        for (int j = 0; j < NB; ++j) b[set][j] = *reinterpret_cast<const bf16x8*>(tile + offB + j * 32 * ROWB + pos);
    };
    auto multiply = [&](int set) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[set][i], b[set][j], acc[i][j], 0, 0, 0);
    };
    // one LDS read after each of the first MB + NB matrix instructions of a slice, the rest of the slice without
    auto pattern = [&]() {
#pragma unroll
        for (int g = 0; g < MB + NB; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // a matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // an LDS read
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MB * NB - (MB + NB), 0);
    };
    request(0, 0);
    request(BK < klast ? BK : klast, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                               // waits for the requests, then for the waves
    operands(lds, 0, 0);
    int buf = 0;
    for (int k0 = 0; k0 < A.D; k0 += BK, buf ^= 1) {
        const char* const cur = lds + buf * BUF;
        const char* const nxt = lds + (buf ^ 1) * BUF;
        __builtin_amdgcn_sched_barrier(0);
        operands(cur, 1, 1);
        multiply(0);
        pattern();
        operands(cur, 2, 0);
        multiply(1);
        pattern();
        operands(cur, 3, 1);
        multiply(0);
        pattern();
        // A wave's own requests are counted by vmcnt; the barrier's fence does not wait for them (they are loads),
        // so the wait is written out: only then may the other waves read what this wave has requested.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                           // the next tile has arrived in every wave's part,
        request(k0 + 2 * BK < klast ? k0 + 2 * BK : klast, buf);   // and this tile's buffer is free for the one after
        operands(nxt, 0, 0);
        multiply(1);
        pattern();
    }

    // Epilogue: bias, then the tile's half of the head (a tile never straddles V: V is a multiple of BN).  The
    // accumulators hold columns across lanes and rows across registers; stored as they are, an instruction would
    // write 128-byte pieces of two rows.  Each wave instead passes its block through LDS, 32 rows at a time (the
    // operand buffers are free by now), and writes whole row segments of 32 NB floats: 16 bytes per lane.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                // the last (repeated) requests have landed
    __syncthreads();                                               // every wave has read its last operands
    constexpr int WCOLS = 32 * NB, SP = WCOLS + 4;                 // staging pitch in floats: rows 4 apart differ in bank
    float* const stage = reinterpret_cast<float*>(lds) + wave * 32 * SP;
    float* out = n0 < A.V ? A.centre : A.radius;
    const int cwave = (n0 < A.V ? n0 : n0 - A.V) + wn * WCOLS;     // first output column of the wave's block
    float bj[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) bj[j] = A.bias ? A.bias[n0 + wn * WCOLS + j * 32 + lrow] : 0.f;
    constexpr int LPR = WCOLS / 4, RPI = 64 / LPR;                 // lanes per row segment, rows per store instruction
    const int srow = lane / LPR, scol = (lane % LPR) * 4;
#pragma unroll
    for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                stage[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * SP + j * 32 + lrow] = acc[i][j][v] + bj[j];
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 32 / RPI; ++t) {
            const int r = t * RPI + srow;
            const int64_t row = m0 + wm * 32 * MB + i * 32 + r;
            const f32x4 val = *reinterpret_cast<const f32x4*>(&stage[r * SP + scol]);
            if (row < A.N) *reinterpret_cast<f32x4*>(&out[row * A.stride + cwave + scol]) = val;
        }
        __syncthreads();
    }
}

template <int MB, int NB>
hipError_t launch_tile(const HeadArgs& a, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    constexpr int BM = 64 * MB, BN = 64 * NB;
    constexpr size_t lds_bytes = (size_t)2 * (BM + BN) * ROWB;                     // 64 KB or 128 KB of the 160 KB
    static_assert(lds_bytes <= 160 * 1024, "tile does not fit the LDS of a compute unit");
    if (lds_bytes > 64 * 1024) {
        // more than the default limit for dynamic LDS: raised for this kernel once per device (an attribute of the
        // function on the device that is current)
        static std::mutex mu;
        static bool raised[64] = {};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
        std::lock_guard<std::mutex> lock(mu);
        if (!raised[dev]) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&interhead_gemm_kernel<MB, NB>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
            if (e != hipSuccess) return e;
            raised[dev] = true;
        }
    }
    HeadArgs args = a;
    args.row_tiles = (int32_t)((a.N + BM - 1) / BM);
    args.col_tiles = 2 * a.V / BN;
    const unsigned grid = (unsigned)args.row_tiles * (unsigned)args.col_tiles;
    if (ev_start && ev_stop)
        hipExtLaunchKernelGGL((interhead_gemm_kernel<MB, NB>), dim3(grid), dim3(256), lds_bytes, stream, ev_start,
                              ev_stop, 0, args);
    else
        hipLaunchKernelGGL((interhead_gemm_kernel<MB, NB>), dim3(grid), dim3(256), lds_bytes, stream, args);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_interhead(const HeadArgs& args, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop)
{
    if (args.N <= 0) return hipSuccess;
    static_assert(kHeadTileCols == 128, "the small tile is the one the C ABI's shape check is written for");
    if (args.V % 256 == 0 && args.N > 128) return launch_tile<4, 4>(args, stream, ev_start, ev_stop);
    return launch_tile<2, 2>(args, stream, ev_start, ev_stop);
}

}  // namespace ciar
