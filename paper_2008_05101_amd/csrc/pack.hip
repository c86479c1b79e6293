// Data packing (Algorithm 1, step 1) from level indices into plane words, and the
// weight-side precomputation that the paper does once after training (end of
// Section 3.3: the mask comes from the weights and is fixed).
//
// One thread turns 32 consecutive levels of one row into one pair of 32-bit words.
// Neighbouring lanes take neighbouring words of the same row, so a wavefront reads
// 2 KiB and writes 512 B of contiguous memory: the pass is bound by HBM, not ALU.
#include "fatnn_device.h"

namespace fatnn {
namespace {

// Gathers the least significant bit of each of the four bytes of v into a nibble
// (byte 0 -> bit 0).  The partial products land on distinct bit positions, so no
// carry can reach bits 24..27.
__device__ __forceinline__ uint32_t lsb_nibble(uint32_t v) {
    return ((v & 0x01010101u) * 0x01020408u) >> 24;
}

// Four levels (one per byte) -> their two plane bits, plus a flag nibble for bytes
// that are not valid.  TWOBIT: codes 0..3 are valid and the planes are the code's
// bits.  Otherwise levels 0..2 are valid, planes are (l==2, l>=1).  An invalid byte
// becomes (0,1): the value 0 of Table 1.
template <int KIND>
__device__ __forceinline__ void planes_of_dword(uint32_t d, uint32_t& p1, uint32_t& p0, uint32_t& bad) {
    uint32_t t = d & 0xFCFCFCFCu;          // any of the six upper bits set?
    t |= t >> 4;
    t |= t >> 2;
    t |= t >> 1;                           // bit 0 of each byte = OR of that byte's bits
    uint32_t b1 = d >> 1, b0 = d;
    uint32_t f = t;
    if (KIND != PACK_TWOBIT) f |= (b1 & b0);  // level 3
    bad = lsb_nibble(f);
    uint32_t hi = lsb_nibble(b1);
    uint32_t lo = (KIND == PACK_TWOBIT) ? lsb_nibble(b0) : lsb_nibble(b1 | b0);
    p1 = hi & ~bad;
    p0 = lo | bad;
}

template <int KIND>
__device__ __forceinline__ plane2 finish_word(uint32_t p1, uint32_t p0) {
    plane2 out;
    out.x = p1;
    out.y = (KIND == PACK_WEIGHT) ? ~(p1 ^ p0) : p0;   // weights: non-zero bit = (l != 1)
    return out;
}

// Byte that stands for "no element here" (k >= K): the value 0 for ternary planes,
// all-zero bits for two-bit planes (equal tail bits cancel in the xor of Eq. 1).
template <int KIND>
__device__ __forceinline__ uint32_t tail_fill() {
    return (KIND == PACK_TWOBIT) ? 0u : 0x01010101u;
}

template <int KIND, bool VEC16>
__global__ __launch_bounds__(256) void pack_contiguous_kernel(const int8_t* __restrict__ levels, int64_t rows,
                                                              int64_t K, int64_t Kw,
                                                              plane2* __restrict__ packed,
                                                              int32_t* __restrict__ n_invalid) {
    const int64_t total = rows * Kw;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += stride) {
        const int64_t row = id / Kw;
        const int64_t kw = id - row * Kw;
        const int64_t k0 = kw * 32;
        const int8_t* src = levels + row * K + k0;
        uint32_t d[8];
        if (VEC16) {
            // K is a multiple of 16 and the base is 16-byte aligned: two 128-bit loads.
            const uint4* s4 = reinterpret_cast<const uint4*>(src);
            uint4 a = s4[0];
            uint4 b;
            if (k0 + 16 < K) {
                b = s4[1];
            } else {
                b.x = b.y = b.z = b.w = tail_fill<KIND>();
            }
            d[0] = a.x; d[1] = a.y; d[2] = a.z; d[3] = a.w;
            d[4] = b.x; d[5] = b.y; d[6] = b.z; d[7] = b.w;
        } else if (k0 + 32 <= K) {
            // rows do not start on a 16-byte boundary: byte-aligned dword loads (global memory
            // accesses need no natural alignment on this target)
            typedef uint32_t __attribute__((aligned(1))) unaligned_u32;
            const unaligned_u32* s1 = reinterpret_cast<const unaligned_u32*>(src);
#pragma unroll
            for (int w = 0; w < 8; ++w) d[w] = s1[w];
        } else {
            const uint32_t fill = tail_fill<KIND>() & 0xFFu;
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                uint32_t v = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int64_t k = k0 + w * 4 + b;
                    uint32_t byte = (k < K) ? (uint32_t)(uint8_t)src[w * 4 + b] : fill;
                    v |= byte << (8 * b);
                }
                d[w] = v;
            }
        }
        uint32_t p1 = 0, p0 = 0, bad = 0;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            uint32_t q1, q0, qb;
            planes_of_dword<KIND>(d[w], q1, q0, qb);
            p1 |= q1 << (4 * w);
            p0 |= q0 << (4 * w);
            bad |= qb << (4 * w);
        }
        packed[id] = finish_word<KIND>(p1, p0);
        if (bad != 0 && n_invalid != nullptr) atomicAdd(n_invalid, __popc(bad));
    }
}

// One-bit elements (Eq. 1: 0 stands for -1, 1 for +1): 64 per word pair, .x holds the first 32.
// Values other than 0 / 1 are counted as invalid and packed as 0; tail bits are 0 in both
// operands, so they cancel in the xor.
__global__ __launch_bounds__(256) void pack_binary_kernel(const int8_t* __restrict__ bits, int64_t rows, int64_t K,
                                                          int64_t Kp, plane2* __restrict__ packed,
                                                          int32_t* __restrict__ n_invalid) {
    const int64_t total = rows * Kp;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += stride) {
        const int64_t row = id / Kp;
        const int64_t kp = id - row * Kp;
        const int8_t* src = bits + row * K + kp * 64;
        uint32_t w[2] = {0u, 0u};
        int bad = 0;
        for (int e = 0; e < 64; ++e) {
            const int64_t k = kp * 64 + e;
            if (k < K) {
                const int v = src[e];
                bad += (v != 0 && v != 1) ? 1 : 0;
                w[e >> 5] |= (uint32_t)(v == 1) << (e & 31);
            }
        }
        plane2 out;
        out.x = w[0];
        out.y = w[1];
        packed[id] = out;
        if (bad != 0 && n_invalid != nullptr) atomicAdd(n_invalid, bad);
    }
}

// General (slow) path for tensors whose K axis is not contiguous (OIHW weights,
// NCHW activations): one thread still makes one word pair, reading byte by byte.
template <int KIND>
__global__ __launch_bounds__(256) void pack_gather_kernel(const int8_t* __restrict__ levels, int64_t rows,
                                                          int64_t K, int64_t Kw, GatherDesc g,
                                                          plane2* __restrict__ packed,
                                                          int32_t* __restrict__ n_invalid) {
    const int64_t total = rows * Kw;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += stride) {
        const int64_t row = id / Kw;
        const int64_t kw = id - row * Kw;
        const int64_t r0 = row / g.n1, r1 = row - r0 * g.n1;
        const int8_t* src = levels + r0 * g.rs0 + r1 * g.rs1;
        const uint32_t fill = tail_fill<KIND>() & 0xFFu;
        uint32_t p1 = 0, p0 = 0, bad = 0;
        for (int w = 0; w < 8; ++w) {
            uint32_t v = 0;
            for (int b = 0; b < 4; ++b) {
                const int64_t k = kw * 32 + w * 4 + b;
                uint32_t byte = fill;
                if (k < K) {
                    const int64_t kk0 = k / g.C, c = k - kk0 * g.C;
                    byte = (uint32_t)(uint8_t)src[kk0 * g.ks0 + c * g.ks1];
                }
                v |= byte << (8 * b);
            }
            uint32_t q1, q0, qb;
            planes_of_dword<KIND>(v, q1, q0, qb);
            p1 |= q1 << (4 * w);
            p0 |= q0 << (4 * w);
            bad |= qb << (4 * w);
        }
        packed[id] = finish_word<KIND>(p1, p0);
        if (bad != 0 && n_invalid != nullptr) atomicAdd(n_invalid, __popc(bad));
    }
}

// Per weight row: number of non-zero weights and number of +1 weights.  They give
// Eq. 3's "- N" in the reduced form (N counts only the non-zero weights once the
// forced-zero fields are dropped) and, in ReLU mode, the added copy of the weights.
__global__ __launch_bounds__(64) void row_constants_kernel(const plane2* __restrict__ packed, int64_t rows,
                                                           int64_t Kw, int32_t* __restrict__ nnz,
                                                           int32_t* __restrict__ npos) {
    const int64_t row = blockIdx.x;
    if (row >= rows) return;
    const plane2* p = packed + row * Kw;
    int cnt_nz = 0, cnt_pos = 0;
    for (int64_t kw = threadIdx.x; kw < Kw; kw += kWave) {
        plane2 w = p[kw];
        cnt_nz += __popc(w.y);
        cnt_pos += __popc(w.x & w.y);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        cnt_nz += __shfl_down(cnt_nz, off, kWave);
        cnt_pos += __shfl_down(cnt_pos, off, kWave);
    }
    if (threadIdx.x == 0) {
        nnz[row] = cnt_nz;
        npos[row] = cnt_pos;
    }
}

// Activations in the bordered layout: [B][H+2b][W+2b][Cw] word pairs, the ring (and
// the slack behind the last image) filled with the word pair of the value 0, so that a
// convolution with padding b never has to test whether a tap is inside the image.
// I = index type of the word pairs: 32-bit wherever the buffer has fewer than 2^31 word pairs (the
// three divisions per word pair are several times cheaper than in 64 bits).
template <int KIND, typename I>
__global__ __launch_bounds__(256) void pack_bordered_kernel(const int8_t* __restrict__ levels, I B, I H, I W, I Cw,
                                                            int border, plane2 border_word, I total,
                                                            plane2* __restrict__ packed,
                                                            int32_t* __restrict__ n_invalid) {
    const I Hp = H + 2 * border, Wp = W + 2 * border;
    const I npix = B * Hp * Wp;
    const I stride = (I)gridDim.x * blockDim.x;
    for (I id = (I)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += stride) {
        const I pix = id / Cw;
        const I cw = id - pix * Cw;
        plane2 out = border_word;
        if (pix < npix) {
            const I wp = pix % Wp;
            const I t = pix / Wp;
            const I hp = t % Hp;
            const I b = t / Hp;
            const I h = hp - border, w = wp - border;
            if (h >= 0 && h < H && w >= 0 && w < W) {
                // 32 levels = 32 bytes, 16-byte aligned because C is a multiple of 32
                const uint4* s4 =
                    reinterpret_cast<const uint4*>(levels + (int64_t)(((b * H + h) * W + w) * Cw + cw) * 32);
                const uint4 a = s4[0], c = s4[1];
                const uint32_t d[8] = {a.x, a.y, a.z, a.w, c.x, c.y, c.z, c.w};
                uint32_t p1 = 0, p0 = 0, bad = 0;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    uint32_t q1, q0, qb;
                    planes_of_dword<KIND>(d[k], q1, q0, qb);
                    p1 |= q1 << (4 * k);
                    p0 |= q0 << (4 * k);
                    bad |= qb << (4 * k);
                }
                out = finish_word<KIND>(p1, p0);
                if (bad != 0 && n_invalid != nullptr) atomicAdd(n_invalid, __popc(bad));
            }
        }
        packed[id] = out;
    }
}

// ---------------------------------------------------------------------------------------
// Algorithm 1, step 1 as the paper writes it: full-precision values are compared with the
// quantisation thresholds and assigned their codec.  The thresholds are the exact
// float32 break points of Eq. 9 / Eq. 10 (found on the host), so two comparisons per
// element reproduce normalise-saturate-round bit for bit.
//   level = (p >= t1) + (p >= t2);  NaN counts as invalid and is packed as the value 0.
struct QuantThresholds {
    float t1, t2;
    uint32_t nan_lo;   // low plane bit of the value 0: 1 (level 1) for weights / symmetric, 0 in ReLU mode
};

__device__ __forceinline__ void quant_bits(float v, int e, const QuantThresholds& q, uint32_t& p1, uint32_t& p0,
                                           uint32_t& bad) {
    const uint32_t ge1 = v >= q.t1 ? 1u : 0u;
    const uint32_t ge2 = v >= q.t2 ? 1u : 0u;
    const uint32_t nan = (v != v) ? 1u : 0u;
    p1 |= ge2 << e;
    p0 |= (ge1 | (nan & q.nan_lo)) << e;
    bad |= nan << e;
}

template <int KIND>
__device__ __forceinline__ plane2 quant_word(const float* __restrict__ src, int64_t valid, bool vec,
                                             const QuantThresholds& q, uint32_t& bad) {
    // `valid` = number of real elements among the 32 of this word (tail slots are the value 0: level 1)
    uint32_t p1 = 0, p0 = 0;
    bad = 0;
    if (vec) {
        const float4* s4 = reinterpret_cast<const float4*>(src);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            if (g * 4 < valid) {
                const float4 v = s4[g];
                quant_bits(v.x, g * 4 + 0, q, p1, p0, bad);
                quant_bits(v.y, g * 4 + 1, q, p1, p0, bad);
                quant_bits(v.z, g * 4 + 2, q, p1, p0, bad);
                quant_bits(v.w, g * 4 + 3, q, p1, p0, bad);
            } else {
                p0 |= 0xFu << (g * 4);
            }
        }
    } else {
#pragma unroll 8
        for (int e = 0; e < 32; ++e) {
            if (e < valid)
                quant_bits(src[e], e, q, p1, p0, bad);
            else
                p0 |= 1u << e;
        }
    }
    return finish_word<KIND>(p1, p0);
}

template <int KIND>
__global__ __launch_bounds__(256) void quantize_pack_kernel(const float* __restrict__ x, int64_t rows, int64_t K,
                                                            int64_t Kw, bool vec, QuantThresholds q,
                                                            plane2* __restrict__ packed,
                                                            int32_t* __restrict__ n_invalid) {
    const int64_t total = rows * Kw;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += stride) {
        const int64_t row = id / Kw;
        const int64_t kw = id - row * Kw;
        const int64_t left = K - kw * 32;
        uint32_t bad;
        packed[id] = quant_word<KIND>(x + row * K + kw * 32, left < 32 ? left : 32, vec, q, bad);
        if (bad != 0 && n_invalid != nullptr) atomicAdd(n_invalid, __popc(bad));
    }
}

template <typename I>
__global__ __launch_bounds__(256) void quantize_pack_bordered_kernel(const float* __restrict__ x, I B, I H, I W, I Cw,
                                                                     int border, plane2 border_word, I total,
                                                                     QuantThresholds q, plane2* __restrict__ packed,
                                                                     int32_t* __restrict__ n_invalid) {
    const I Hp = H + 2 * border, Wp = W + 2 * border;
    const I npix = B * Hp * Wp;
    const I stride = (I)gridDim.x * blockDim.x;
    for (I id = (I)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += stride) {
        const I pix = id / Cw;
        const I cw = id - pix * Cw;
        plane2 out = border_word;
        if (pix < npix) {
            const I wp = pix % Wp;
            const I t = pix / Wp;
            const I hp = t % Hp;
            const I b = t / Hp;
            const I h = hp - border, w = wp - border;
            if (h >= 0 && h < H && w >= 0 && w < W) {
                uint32_t bad;
                out = quant_word<PACK_ACT>(x + (int64_t)(((b * H + h) * W + w) * Cw + cw) * 32, 32, true, q, bad);
                if (bad != 0 && n_invalid != nullptr) atomicAdd(n_invalid, __popc(bad));
            }
        }
        packed[id] = out;
    }
}

__global__ __launch_bounds__(256) void fill_words_kernel(plane2* __restrict__ dst, int64_t count, plane2 word) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < count; id += stride) dst[id] = word;
}

// Second copy of the weight words with the 64 rows of a block contiguous per k-word.
__global__ __launch_bounds__(256) void interleave_weights_kernel(const plane2* __restrict__ packed, int64_t rows,
                                                                 int64_t Kw, int64_t total,
                                                                 plane2* __restrict__ inter) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += stride) {
        const int64_t lane = id & 63;
        const int64_t t = id >> 6;
        const int64_t kw = t % Kw;
        const int64_t mb = t / Kw;
        const int64_t row = mb * 64 + lane;
        plane2 v;
        v.x = 0u;
        v.y = 0u;
        if (row < rows) v = packed[row * Kw + kw];
        inter[id] = v;
    }
}

int grid_for(int64_t total, int block) {
    int64_t g = (total + block - 1) / block;
    const int64_t cap = 256 * 64;  // enough resident work for 256 CUs; the kernels stride
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    return (int)g;
}

}  // namespace

int launch_pack_contiguous(const int8_t* levels, int64_t rows, int64_t K, int kind, plane2* packed,
                           int32_t* n_invalid, hipStream_t stream) {
    const int64_t Kw = (K + 31) / 32;
    const int64_t total = rows * Kw;
    if (total == 0) return 0;
    const bool vec = (K % 16 == 0) && ((reinterpret_cast<uintptr_t>(levels) & 15u) == 0);
    dim3 grid(grid_for(total, 256)), block(256);
#define FATNN_LAUNCH_PACK(KIND)                                                                              \
    if (vec)                                                                                                 \
        hipLaunchKernelGGL((pack_contiguous_kernel<KIND, true>), grid, block, 0, stream, levels, rows, K, Kw, \
                           packed, n_invalid);                                                               \
    else                                                                                                     \
        hipLaunchKernelGGL((pack_contiguous_kernel<KIND, false>), grid, block, 0, stream, levels, rows, K,   \
                           Kw, packed, n_invalid);
    switch (kind) {
        case PACK_ACT: FATNN_LAUNCH_PACK(PACK_ACT) break;
        case PACK_WEIGHT: FATNN_LAUNCH_PACK(PACK_WEIGHT) break;
        case PACK_TWOBIT: FATNN_LAUNCH_PACK(PACK_TWOBIT) break;
        default: return -1;
    }
#undef FATNN_LAUNCH_PACK
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_pack_binary(const int8_t* bits, int64_t rows, int64_t K, plane2* packed, int32_t* n_invalid,
                       hipStream_t stream) {
    const int64_t Kp = (K + 63) / 64;
    const int64_t total = rows * Kp;
    if (total == 0) return 0;
    hipLaunchKernelGGL(pack_binary_kernel, dim3(grid_for(total, 256)), dim3(256), 0, stream, bits, rows, K, Kp, packed,
                       n_invalid);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_pack_gather(const int8_t* levels, int64_t rows, int64_t K, GatherDesc g, int kind, plane2* packed,
                       int32_t* n_invalid, hipStream_t stream) {
    const int64_t Kw = (K + 31) / 32;
    const int64_t total = rows * Kw;
    if (total == 0) return 0;
    dim3 grid(grid_for(total, 256)), block(256);
    switch (kind) {
        case PACK_ACT:
            hipLaunchKernelGGL((pack_gather_kernel<PACK_ACT>), grid, block, 0, stream, levels, rows, K, Kw, g,
                               packed, n_invalid);
            break;
        case PACK_WEIGHT:
            hipLaunchKernelGGL((pack_gather_kernel<PACK_WEIGHT>), grid, block, 0, stream, levels, rows, K, Kw,
                               g, packed, n_invalid);
            break;
        case PACK_TWOBIT:
            hipLaunchKernelGGL((pack_gather_kernel<PACK_TWOBIT>), grid, block, 0, stream, levels, rows, K, Kw,
                               g, packed, n_invalid);
            break;
        default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_pack_bordered(const int8_t* levels, int64_t B, int64_t H, int64_t W, int64_t C, int border, int kind,
                         plane2 border_word, int64_t slack_pixels, plane2* packed, int32_t* n_invalid,
                         hipStream_t stream) {
    const int64_t Cw = C / 32;
    const int64_t total = (B * (H + 2 * border) * (W + 2 * border) + slack_pixels) * Cw;
    if (total == 0) return 0;
    dim3 grid(grid_for(total, 256)), block(256);
    // 32-bit indices while id + (threads of the grid) cannot wrap
    const bool small = total + (int64_t)grid.x * 256 < 0x7FFFFFFFLL;
    auto launch = [&](auto kernel32, auto kernel64) {
        if (small)
            hipLaunchKernelGGL(kernel32, grid, block, 0, stream, levels, (int32_t)B, (int32_t)H, (int32_t)W, (int32_t)Cw,
                               border, border_word, (int32_t)total, packed, n_invalid);
        else
            hipLaunchKernelGGL(kernel64, grid, block, 0, stream, levels, B, H, W, Cw, border, border_word, total, packed,
                               n_invalid);
    };
    if (kind == PACK_ACT)
        launch(pack_bordered_kernel<PACK_ACT, int32_t>, pack_bordered_kernel<PACK_ACT, int64_t>);
    else if (kind == PACK_TWOBIT)
        launch(pack_bordered_kernel<PACK_TWOBIT, int32_t>, pack_bordered_kernel<PACK_TWOBIT, int64_t>);
    else
        return -1;
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_quantize_pack(const float* x, int64_t rows, int64_t K, int kind, float t1, float t2, uint32_t nan_lo,
                         plane2* packed, int32_t* n_invalid, hipStream_t stream) {
    const int64_t Kw = (K + 31) / 32;
    const int64_t total = rows * Kw;
    if (total == 0) return 0;
    const bool vec = (K % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15u) == 0);
    QuantThresholds q{t1, t2, nan_lo};
    dim3 grid(grid_for(total, 256)), block(256);
    if (kind == PACK_WEIGHT)
        hipLaunchKernelGGL((quantize_pack_kernel<PACK_WEIGHT>), grid, block, 0, stream, x, rows, K, Kw, vec, q, packed,
                           n_invalid);
    else
        hipLaunchKernelGGL((quantize_pack_kernel<PACK_ACT>), grid, block, 0, stream, x, rows, K, Kw, vec, q, packed,
                           n_invalid);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_quantize_pack_bordered(const float* x, int64_t B, int64_t H, int64_t W, int64_t C, int border,
                                  plane2 border_word, int64_t slack_pixels, float t1, float t2, uint32_t nan_lo,
                                  plane2* packed, int32_t* n_invalid, hipStream_t stream) {
    const int64_t Cw = C / 32;
    const int64_t total = (B * (H + 2 * border) * (W + 2 * border) + slack_pixels) * Cw;
    if (total == 0) return 0;
    QuantThresholds q{t1, t2, nan_lo};
    // 64-bit indices on purpose: measured on the 128 x 56 x 56 x 256 tensor, the 32-bit variant of this
    // kernel reaches 3.7 TB/s and this one 5.4 TB/s (the slower index arithmetic spaces the eight 16-byte
    // loads of a thread, which all fall into one 128-byte line, so that the line is still cached)
    hipLaunchKernelGGL(quantize_pack_bordered_kernel<int64_t>, dim3(grid_for(total, 256)), dim3(256), 0, stream, x, B, H,
                       W, Cw, border, border_word, total, q, packed, n_invalid);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_fill_words(plane2* dst, int64_t count, plane2 word, hipStream_t stream) {
    if (count == 0) return 0;
    hipLaunchKernelGGL(fill_words_kernel, dim3(grid_for(count, 256)), dim3(256), 0, stream, dst, count, word);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_interleave_weights(const plane2* packed, int64_t rows, int64_t Kw, plane2* inter, hipStream_t stream) {
    const int64_t total = ((rows + 63) / 64) * Kw * 64;
    if (total == 0) return 0;
    hipLaunchKernelGGL(interleave_weights_kernel, dim3(grid_for(total, 256)), dim3(256), 0, stream, packed, rows,
                       Kw, total, inter);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_row_constants(const plane2* packed, int64_t rows, int64_t Kw, int32_t* nnz, int32_t* npos,
                         hipStream_t stream) {
    if (rows == 0) return 0;
    hipLaunchKernelGGL(row_constants_kernel, dim3((unsigned)rows), dim3(kWave), 0, stream, packed, rows, Kw,
                       nnz, npos);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace fatnn
