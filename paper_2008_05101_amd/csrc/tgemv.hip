// Ternary GEMM with few columns (fully connected layers at small batch; the paper treats them as
// convolutions whose kernel covers the whole feature map, Supplementary S1): matrix-vector shaped,
// bound by streaming the packed weights.  A wavefront owns RW weight rows; its 64 lanes split K
// (lane l takes k-words l, l+64, ...), so every load of a weight row is one contiguous 512-byte
// request.  Per k-word the lane evaluates the same reduced form of Eq. 3 as the tiled kernel
// (2 logic + 2 popcount instructions per word pair and column); a butterfly over the lanes then
// sums the partial popcounts.  More than NC columns are done NC at a time; the wavefront's weight
// rows (a few KB) come from L1 again for every chunk.
#include "fatnn_device.h"

namespace fatnn {
namespace {

constexpr int RW = 4;   // weight rows per wavefront

__device__ __forceinline__ void popc_acc(int32_t& acc, uint32_t x) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

template <int NC>
__global__ __launch_bounds__(256) void skinny_gemm_kernel(const GemmParams p) {
    const int lane = threadIdx.x & 63;
    const int wave = (int)((blockIdx.x * (blockDim.x >> 6)) + (threadIdx.x >> 6));
    const int m0 = wave * RW;
    if (m0 >= p.M) return;

  for (int n0 = 0; n0 < p.N; n0 += NC) {
    int32_t acc[RW][NC];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[r][c] = 0;

    for (int kw = lane; kw < p.Kw; kw += 64) {
        plane2 a[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            a[c].x = 0u;
            a[c].y = 0u;
            if (n0 + c < p.N) a[c] = p.A[(int64_t)(n0 + c) * p.Kw + kw];
        }
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            plane2 w;
            w.x = 0u;
            w.y = 0u;   // a row past M is all-zero weights
            if (m0 + r < p.M) w = p.W[(int64_t)(m0 + r) * p.Kw + kw];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                popc_acc(acc[r][c], (a[c].x ^ w.x) & w.y);
                popc_acc(acc[r][c], (a[c].y ^ w.x) & w.y);
            }
        }
    }
    // sum over the 64 lanes
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            int32_t v = acc[r][c];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            acc[r][c] = v;
        }
    // lane (r * NC + c) writes output (m0 + r, c)
    if (lane < RW * NC) {
        const int r = lane / NC, c = lane % NC;
        int32_t sum = 0;
#pragma unroll
        for (int rr = 0; rr < RW; ++rr)
#pragma unroll
            for (int cc = 0; cc < NC; ++cc)
                if (rr == r && cc == c) sum = acc[rr][cc];
        const int m = m0 + r;
        const int n = n0 + c;
        if (m < p.M && n < p.N) {
            const int32_t v = p.cmul * p.rowc[m] - sum;
            if (p.C != nullptr) p.C[(int64_t)m * p.ldc_m + (int64_t)n * p.ldc_n] = v;
            if (p.Cf != nullptr) {
                float f = p.scale[m] * (float)v;
                if (p.bias != nullptr) f = f + p.bias[m];
                p.Cf[(int64_t)m * p.ldf_m + (int64_t)n * p.ldf_n] = f;
            }
        }
    }
  }
}

}  // namespace

// Up to four columns, and up to eight with a short K.  Measured for M = 4096, K = 4608: 3.7 / 4.4 / 5.5 / 7.6 us
// at N = 1 / 2 / 4 / 8; the K-splitting kernel of the tiled family takes 6.1 us for any N up to 32 there (and
// 18.5 against this kernel's 17.8 us at 1000 x 8 x 25088), so it serves five columns and more when K >= 2048.
bool skinny_supported(const GemmParams& p, int op) {
    if (op != OP_TERNARY || p.is_conv) return false;
    return p.N <= 4 || (p.N <= 8 && p.Kw < 64);
}

int launch_skinny_gemm(const GemmParams& p, hipStream_t stream) {
    const int waves = (p.M + RW - 1) / RW;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    const LaunchTiming t = take_launch_timing();
    if (p.N <= 1)
        hipExtLaunchKernelGGL((skinny_gemm_kernel<1>), dim3(grid), dim3(256), 0, stream, t.start, t.stop, 0, p);
    else if (p.N <= 2)
        hipExtLaunchKernelGGL((skinny_gemm_kernel<2>), dim3(grid), dim3(256), 0, stream, t.start, t.stop, 0, p);
    else if (p.N <= 4)
        hipExtLaunchKernelGGL((skinny_gemm_kernel<4>), dim3(grid), dim3(256), 0, stream, t.start, t.stop, 0, p);
    else
        hipExtLaunchKernelGGL((skinny_gemm_kernel<8>), dim3(grid), dim3(256), 0, stream, t.start, t.stop, 0, p);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace fatnn
