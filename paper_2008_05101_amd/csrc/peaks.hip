// Measurement kernels that fix the denominators of the roofline report on the chip itself.
//
// (1) VALU issue rate of the method's own instruction pair.  The reduced form of Eq. 3
//     (Section 3.3) costs one three-input logic instruction and one accumulating popcount per
//     32-bit plane word; valu_probe_kernel issues exactly that pair (or one of its halves) from
//     registers only, with a chosen number of wavefronts per SIMD, so that
//         lane-instructions / second = blocks * 256 * iters * kPairsPerIter * 2 / time
//     is the rate at which the arithmetic of the GEMM / convolution kernels could run if operand
//     delivery were free.  It is a ceiling for them by construction: same instructions, same
//     dependent logic -> popcount ordering, no memory traffic.
// (2) HBM streaming rate: a read-only, a write-only and a copy pass over a large buffer with
//     128-bit accesses, every access coalesced.
//
// Nothing here is on the product path.
#include "fatnn_device.h"

namespace fatnn {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeWords = 8;                       // x words held in registers
constexpr int kProbeAccs = 8;                        // accumulators (chains)
constexpr int kPairsPerIter = kProbeWords * kProbeAccs;

enum : int { PROBE_PAIR_V = 0, PROBE_PAIR_S = 1, PROBE_BCNT = 2, PROBE_BITOP3 = 3, PROBE_XOR = 4, PROBE_PAIR_LDS = 5 };

// KIND  PROBE_PAIR_V  logic (all-VGPR operands) feeding the popcount of the same accumulator chain,
//                     the ordering the tiled GEMM kernel uses
//       PROBE_PAIR_S  the same with the data word in an SGPR, as the column-streaming kernel issues it
//       PROBE_BCNT    the popcount alone, PROBE_BITOP3 the logic instruction alone, PROBE_XOR a plain
//                     two-input VOP2 (for reference)
//       PROBE_PAIR_LDS the pair with its data words re-read from LDS at the large GEMM tile's ratio (one
//                     128-bit read per 16 pairs, issued one half-iteration ahead of its use): what operand
//                     delivery through LDS alone costs, without global loads, barriers or address arithmetic
template <int KIND>
__global__ __launch_bounds__(256) void valu_probe_kernel(const int iters, const uint32_t* __restrict__ seed,
                                                        int32_t* __restrict__ sink) {
    const int tid = threadIdx.x;
    uint32_t x[kProbeWords], sx[kProbeWords];
#pragma unroll
    for (int i = 0; i < kProbeWords; ++i) {
        x[i] = seed[(tid + 64 * i) & 1023];
        sx[i] = __builtin_amdgcn_readfirstlane(seed[(i + blockIdx.x) & 1023]);
    }
    uint32_t s = seed[(tid + 7) & 1023], nm = seed[(tid + 300) & 1023];
    int32_t acc[kProbeAccs];
#pragma unroll
    for (int a = 0; a < kProbeAccs; ++a) acc[a] = 0;
    uint32_t t = 0;
    if constexpr (KIND == PROBE_PAIR_LDS) {
        __shared__ __attribute__((aligned(16))) uint32_t tile[256 * 4 * 2];
        for (int i = 0; i < 8; ++i) tile[tid * 8 + i] = x[i];
        __syncthreads();
        // eight distinct 16-byte addresses per wavefront and read, as in the tile kernel's fragment reads
        const uint4* src = reinterpret_cast<const uint4*>(tile) + (tid & 56);
        uint4 nx0 = src[0], nx1 = src[1];
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const uint4 c0 = nx0, c1 = nx1;
                nx0 = src[(2 * it + half) & 7];          // in flight while the 32 pairs below issue
                nx1 = src[((2 * it + half) & 7) + 256];
                const uint32_t xs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
                FATNN_VOP3_RUN_PHASE();
#pragma unroll
                for (int a = 0; a < 4; ++a) {
#pragma unroll
                    for (int i = 0; i < kProbeWords; ++i) {
                        asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x48" : "=v"(t) : "v"(xs[i]), "v"(s), "v"(nm));
                        asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[half * 4 + a]) : "v"(t));
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        t ^= nx0.x ^ nx1.x;
    } else
    for (int it = 0; it < iters; ++it) {
        FATNN_VOP3_RUN_PHASE();
#pragma unroll
        for (int a = 0; a < kProbeAccs; ++a) {
#pragma unroll
            for (int i = 0; i < kProbeWords; ++i) {
                if constexpr (KIND == PROBE_PAIR_V) {
                    asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x48" : "=v"(t) : "v"(x[i]), "v"(s), "v"(nm));
                    asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[a]) : "v"(t));
                } else if constexpr (KIND == PROBE_PAIR_S) {
                    asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x48" : "=v"(t) : "s"(sx[i]), "v"(s), "v"(nm));
                    asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[a]) : "v"(t));
                } else if constexpr (KIND == PROBE_BCNT) {
                    asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[a]) : "v"(x[i]));
                    asm volatile("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc[a]) : "v"(s));
                } else if constexpr (KIND == PROBE_BITOP3) {
                    asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x48" : "=v"(t) : "v"(x[i]), "v"(s), "v"(nm));
                    asm volatile("v_bitop3_b32 %0, %1, %2, %3 bitop3:0x48"
                                 : "=v"(acc[a])
                                 : "v"(x[i]), "v"(nm), "v"(s));
                } else {
                    asm volatile("v_xor_b32 %0, %1, %2" : "=v"(t) : "v"(x[i]), "v"(s));
                    asm volatile("v_xor_b32 %0, %1, %2" : "=v"(acc[a]) : "v"(x[i]), "v"(nm));
                }
            }
        }
    }
    int32_t r = (int32_t)t;
#pragma unroll
    for (int a = 0; a < kProbeAccs; ++a) r += acc[a];
    sink[(size_t)blockIdx.x * 256 + tid] = r;
}

// Streaming passes over n 16-byte words.  Every workgroup walks the buffer with the whole grid's stride,
// so all accesses of a moment fall into one compact window.
__global__ __launch_bounds__(256) void hbm_read_kernel(const u32x4* __restrict__ src, const size_t n,
                                                      uint32_t* __restrict__ sink) {
    uint32_t a = 0;
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        a ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // one word per thread keeps the loads alive; 1/1000 of the traffic or less
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = a;
}

// Stores through a buffer resource with the policy device scope + non-temporal, the one the convolution
// kernels' output stores use (measured there: faster than plain or non-temporal-only stores).  The buffer is
// below 4 GiB (the host checks).
__global__ __launch_bounds__(256) void hbm_write_kernel(u32x4* __restrict__ dst, const size_t n) {
    constexpr int kRsrcFlags = 0x00020000;
    constexpr int kStreamOut = 16 | 2;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(dst, 0, (int)(uint32_t)(n * 16), kRsrcFlags);
    const size_t stride = (size_t)gridDim.x * 256;
    const u32x4 v = {0x01010101u, 0x02020202u, 0x03030303u, (uint32_t)blockIdx.x};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
        __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, (int)(uint32_t)(i * 16), 0, kStreamOut);
}

__global__ __launch_bounds__(256) void hbm_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                      const size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

int probe_pairs_per_iteration() { return kPairsPerIter; }

int launch_valu_probe(int kind, int blocks, int iters, const uint32_t* seed, int32_t* sink, hipStream_t stream) {
    const LaunchTiming t = take_launch_timing();
#define FATNN_PROBE_CASE(K)                                                                                    \
    case K:                                                                                                    \
        hipExtLaunchKernelGGL((valu_probe_kernel<K>), dim3(blocks), dim3(256), 0, stream, t.start, t.stop, 0,   \
                              iters, seed, sink);                                                              \
        break;
    switch (kind) {
        FATNN_PROBE_CASE(PROBE_PAIR_V)
        FATNN_PROBE_CASE(PROBE_PAIR_S)
        FATNN_PROBE_CASE(PROBE_BCNT)
        FATNN_PROBE_CASE(PROBE_BITOP3)
        FATNN_PROBE_CASE(PROBE_XOR)
        FATNN_PROBE_CASE(PROBE_PAIR_LDS)
        default: return -3;
    }
#undef FATNN_PROBE_CASE
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_hbm_probe(int kind, void* dst, const void* src, size_t bytes, int blocks, uint32_t* sink,
                     hipStream_t stream) {
    const LaunchTiming t = take_launch_timing();
    const size_t n = bytes / sizeof(u32x4);
    if (kind == 0)
        hipExtLaunchKernelGGL(hbm_read_kernel, dim3(blocks), dim3(256), 0, stream, t.start, t.stop, 0,
                              reinterpret_cast<const u32x4*>(src), n, sink);
    else if (kind == 1)
        hipExtLaunchKernelGGL(hbm_write_kernel, dim3(blocks), dim3(256), 0, stream, t.start, t.stop, 0,
                              reinterpret_cast<u32x4*>(dst), n);
    else if (kind == 2)
        hipExtLaunchKernelGGL(hbm_copy_kernel, dim3(blocks), dim3(256), 0, stream, t.start, t.stop, 0,
                              reinterpret_cast<u32x4*>(dst), reinterpret_cast<const u32x4*>(src), n);
    else
        return -3;
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace fatnn
