// Weight-stationary, column-streaming convolution kernels for gfx950.
//
// Convolution layers of CNNs have few output channels (64..512), a short K per
// output (R*S*Cin <= a few thousand) and very many columns (batch x pixels).  Here
// a wavefront keeps packed weights of 64 output channels in VGPRs for its whole
// life (lane = output channel) and walks over groups of U neighbouring output
// pixels.  The activation plane words of a pixel are the same for every lane, so
// they are fetched with scalar loads into SGPRs and enter the three-input logic
// instruction as its scalar operand: no LDS and no barrier in the K loop, and the
// work of a wavefront can be any number of groups, which removes the tile
// quantisation that small layers suffer on 256 CUs.
//
// The scalar cache serves roughly one request per 15 clocks per CU whatever the
// request size, so the kernel reads 64-byte requests where it can and re-uses
// every fetched input pixel for all the (output pixel, filter tap) pairs of the
// group that touch it: an image-row strip of (U-1)*stride + R input pixels serves
// U output pixels.  The input must be the bordered layout (physical ring of
// value-0 pixels, slack behind the last image), so strips never need a bounds check.
//
// What was measured on the chip and shaped the rest (details at the places):
//  * a wavefront holds at most four channel words of every tap; wider layers are
//    split over two or four wavefronts per block of 64 channels that meet in LDS
//    once per group (more wavefronts per SIMD beat fewer, larger ones);
//  * wavefronts lower their own priority towards their end, so the wavefronts of a
//    SIMD finish together instead of one after the other;
//  * the ranges that get one group more are the first in dispatch order, which
//    spreads them over the SIMDs; for the write-heavy shapes a wavefront takes
//    every n-th group, so that the output is written as one compact front;
//  * outputs are stored through buffer resources (no vector address arithmetic)
//    with device scope + non-temporal policy.
//
// The arithmetic is the reduced form of Eq. 3 (Section 3.3): 2 logic + 2 popcount
// instructions per 32 elements; the two-bit form of Eq. 2 needs 4 + 4.
#include "fatnn_device.h"

#include <atomic>
#include <type_traits>
#include <utility>

namespace fatnn {
namespace {

typedef const __attribute__((address_space(4))) uint32_t* sptr_t;   // scalar-loadable (constant) memory
typedef const __attribute__((address_space(4))) char* sbytes_t;

__device__ __forceinline__ void popc_acc(int32_t& acc, uint32_t x) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

// v[LANE] = s for a wave-uniform s; the other lanes keep their value.
template <int LANE>
__device__ __forceinline__ void write_lane(uint32_t& v, uint32_t s) {
    asm("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(s), "n"(LANE));
}

// Wave-uniform load of NW consecutive dwords through the scalar cache (dword alignment suffices).
template <int NW>
__device__ __forceinline__ void sload(const sptr_t src, uint32_t* dst) {
    typedef uint32_t vec_t __attribute__((ext_vector_type(NW)));
    typedef const __attribute__((address_space(4))) vec_t* vptr_t;
    const vec_t v = *reinterpret_cast<vptr_t>(src);
#pragma unroll
    for (int i = 0; i < NW; ++i) dst[i] = v[i];
}

// ND consecutive dwords as the fewest scalar requests (16, 8, 4, 2 dwords each).
template <int ND, int OFF = 0>
__device__ __forceinline__ void sload_run(const sptr_t src, uint32_t* dst) {
    if constexpr (ND - OFF >= 16) {
        sload<16>(src + OFF, dst + OFF);
        sload_run<ND, OFF + 16>(src, dst);
    } else if constexpr (ND - OFF >= 8) {
        sload<8>(src + OFF, dst + OFF);
        sload_run<ND, OFF + 8>(src, dst);
    } else if constexpr (ND - OFF >= 4) {
        sload<4>(src + OFF, dst + OFF);
        sload_run<ND, OFF + 4>(src, dst);
    } else if constexpr (ND - OFF >= 2) {
        sload<2>(src + OFF, dst + OFF);
        sload_run<ND, OFF + 2>(src, dst);
    }
}

// CW = channel words one wavefront keeps resident, CWT = channel words per stored pixel (CWT = CW * wavefronts
// sharing a row block).
template <int R, int CW, int ST, int U>
struct StreamShape {
    static constexpr int PD = 2 * CW;                        // dwords per packed pixel
    static constexpr int SP = (U - 1) * ST + R;              // input pixels per image-row strip
    // pixels per batch: one 64-byte request where possible, except where a slightly different
    // size makes the number of batches per group even (an odd number needs the group body twice,
    // once per buffer parity, and the doubled code costs instruction-cache misses at kernel start)
    static constexpr int PB = (R == 3 && CW == 4 && ST == 1 && U == 4)   ? 3
                              : (R == 3 && CW == 2 && ST == 1 && U == 8) ? 5
                              : (R == 3 && CW == 2 && ST == 2 && U == 4) ? 5
                              : ((16 / PD) > 0 ? (16 / PD) : 1);
    static constexpr int CH = (SP + PB - 1) / PB;            // batches per strip
    static constexpr int NBATCH = R * CH;                    // batches per group
    static constexpr int BUF = PB * PD;                      // dwords per batch buffer
};

// What happens to the finished sums: EPI_PLAIN writes int32 (and/or scaled fp32) NHWC outputs;
// EPI_CHAIN applies the fused layer epilogue and writes the next layer's packed input.
enum : int { EPI_PLAIN = 0, EPI_CHAIN = 1 };

// KH = CWT / CW wavefronts share a (row block, range) when one wavefront does not hold all channel words:
// each keeps CW of the CWT channel words of every tap and sums over its part of K; at the end of every
// group the partial sums of the wavefronts 1 .. KH-1 go through LDS to wavefront 0, which runs the epilogue.
template <int OP, int R, int CW, int CWT, int ST, int U, int EPI>
__global__ __launch_bounds__(256 * (CWT / CW)) void stream_conv_kernel(const StreamParams p) {
    typedef StreamShape<R, CW, ST, U> Sh;
    constexpr int TAPS = R * R, PD = Sh::PD, SP = Sh::SP, PB = Sh::PB, CH = Sh::CH, NBATCH = Sh::NBATCH;
    constexpr int KH = CWT / CW;
    static_assert(CWT % CW == 0, "the wavefronts of a row block split the channel words evenly");
    // hand-over of partial sums (KH > 1 only): [row block of the workgroup][group parity][pixel][lane]
    extern __shared__ int32_t handover[];
    // Every wavefront starts at the priority its first groups run at: one that loaded its weights at the
    // default (lowest) priority next to older wavefronts already in their groups was starved by them and
    // reached its own first group up to 20 us late (measured), which left the SIMD with too few wavefronts
    // at the end.
    __builtin_amdgcn_s_setprio(3);
    const int lane = threadIdx.x & 63;
    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kh = KH > 1 ? wave_in_block % KH : 0;   // this wavefront's part of K
    const int mbl = wave_in_block / KH;               // row block inside the workgroup
    // One-dimensional grid: workgroup = (range of groups, set of row blocks), the row-block set
    // varying fastest, so that in dispatch order the ranges come one after the other.
    const int wpb = (blockDim.x >> 6) / KH;           // row blocks per workgroup
    const int mblocks = (p.M + 63) / 64;
    const int nsets = (mblocks + wpb - 1) / wpb;
    const int range = blockIdx.x / nsets;
    int mb = (blockIdx.x - range * nsets) * wpb + mbl;
    if (KH == 1) {
        if (mb >= mblocks) return;
    } else if (mb >= mblocks) {
        // every wavefront of the workgroup must reach the barriers: a surplus wavefront repeats
        // the last row block (and stores the same values a second time)
        mb = mblocks - 1;
    }
    // Lanes past the last output channel (M not a multiple of 64) take the last channel's
    // constants and output slot: they compute and store a duplicate of that channel, which
    // saves every per-lane mask in the epilogues; only the quantizer ballots drop their bits.
    const int m_real = mb * 64 + lane;
    const bool m_ok = m_real < p.M;
    const int m = m_ok ? m_real : p.M - 1;
    const uint64_t ok_mask = __ballot(m_ok);

    plane2 w[TAPS][CW];   // this wavefront's weights of the lane's output channel
    const plane2* wsrc = p.Wi + ((int64_t)mb * p.Kw) * 64 + (m - mb * 64);   // duplicates read the last channel's weights
    // The row constant is loaded here but multiplied only in the epilogue: arithmetic on it in
    // the prologue would make every wavefront wait out a memory round trip before it even
    // requests its weights.
    int32_t rc_raw = 0;
    // a missing bias (and a missing skip value below) is -0.0f: x + (-0.0f) == x bit for bit for
    // every x, so the additions need no condition
    float neg0 = -0.0f;
    // one register for the constant instead of re-materialising it per use, where registers are not scarce
    if constexpr (CW < 8) asm volatile("" : "+v"(neg0));
    float sc = 0.f, bs = neg0;
    if (OP == OP_TERNARY) rc_raw = p.rowc[m];
    if (EPI == EPI_CHAIN || p.Cf != nullptr) {
        sc = p.scale[m];
        if (p.bias != nullptr) bs = p.bias[m];
    }

    // ---- this wavefront's range of groups; a group = U neighbouring pixels of one output row.
    // Range r owns gq + (r < gr) groups: the ranges that get one group more are the first ones
    // in dispatch order, which the hardware spreads over the compute units (a stride between
    // them would put them all on the same SIMDs and make those finish a whole group late).
    const int g_begin = range * p.gq + (range < p.gr ? range : p.gr);
    const int count = p.gq + (range < p.gr ? 1 : 0);
    if (count == 0) return;

    // All positions are 32-bit offsets that advance from group to group (the host checks that
    // the input, the outputs and the next layer's buffer are each smaller than 4 GiB).
    const int wgroups = p.wgroups;
    constexpr uint32_t kPixBytes = CWT * 8u;
    constexpr uint32_t kInStep = (uint32_t)(U * ST) * kPixBytes;
    const uint32_t row_bytes = (uint32_t)p.Wp * kPixBytes;
    const uint32_t img_bytes = (uint32_t)p.Hp * row_bytes;
    const uint32_t in_row_adj = (uint32_t)ST * row_bytes - (uint32_t)(wgroups - 1) * kInStep;
    const uint32_t in_img_adj = img_bytes - (uint32_t)((p.Ho - 1) * ST) * row_bytes - (uint32_t)(wgroups - 1) * kInStep;
    const uint32_t ldc = (uint32_t)p.ldc;
    const uint32_t out_step = (uint32_t)U * ldc, out_tail = (uint32_t)p.tailU * ldc;
    const uint32_t nx_step = (uint32_t)(U * p.nCw);
    const uint32_t nx_row_adj = (uint32_t)((p.nWp - (wgroups - 1) * U) * p.nCw);
    const uint32_t nx_img_adj = (uint32_t)(((p.nHp - p.Ho + 1) * p.nWp - (wgroups - 1) * U) * p.nCw);

    int wg, ho;                 // group in the output row, output row in the image
    uint32_t goff;              // byte offset of the group's first strip in the bordered input
    uint32_t ooff;              // element offset of the group's first output pixel, channel 0
    uint32_t noff = 0;          // word-pair offset of that pixel in the next layer's bordered input
    // 1x1 filters (and the 3x3 shapes listed below): a wavefront takes every nranges-th group instead
    // of a contiguous block, so that
    // all wavefronts move through the output as one compact front.  These layers are bound by
    // writing their output, and 1000 separate write streams reach 5.0 TB/s on this chip where a
    // compact front reaches 5.9 (measured with a store-only kernel of the same pattern); with a
    // 1x1 filter neighbouring groups share no input, so nothing is lost on the read side.
    // Measured per shape: it also pays for the 64-channel 3x3 layers (35.5 -> 33 us, stride 2: 21.2 -> 18.4)
    // and a little for the 128-channel stride-1 ones; the 256-channel layers lose 2-3 us with it.
    constexpr bool kStrided = (R == 1 && ST == 1) || (R == 3 && (CW == 2 || (CW == 4 && ST == 1)));
    int img = 0;                // image of the current group (strided walk only)
    const int Wo = (wgroups - 1) * U + p.tailU;
    auto locate = [&]() {       // offsets of group (img, ho, wg)
        goff = (uint32_t)img * img_bytes + (uint32_t)(ho * ST + p.xoff) * row_bytes +
               (uint32_t)(wg * U * ST + p.xoff) * kPixBytes;
        ooff = (uint32_t)((img * p.Ho + ho) * Wo + wg * U) * ldc;
        if (EPI == EPI_CHAIN)
            noff = (uint32_t)(((img * p.nHp + ho + p.nborder) * p.nWp + wg * U + p.nborder) * p.nCw);
    };
    auto seek = [&]() {
        const int g0 = kStrided ? range : g_begin;
        wg = g0 % wgroups;
        const int t0 = g0 / wgroups;
        ho = t0 % p.Ho;
        img = t0 / p.Ho;
        locate();
    };
    // the stride of the strided walk, split into (images, rows, groups)
    const int nranges = kStrided ? (int)(gridDim.x / nsets) : 1;
    const int step_wg = nranges % wgroups;
    const int step_ho = (nranges / wgroups) % p.Ho;
    const int step_img = (nranges / wgroups) / p.Ho;

    const sbytes_t xbase = (sbytes_t)(uintptr_t)p.A + (uint32_t)kh * (CW * 8u);

    // batch i of a group = pixels [c*PB, c*PB+np) of the strip of filter row r
    auto issue = [&](auto i_tag, uint32_t at, uint32_t* dst) {
        constexpr int i = decltype(i_tag)::value;
        constexpr int r = i / CH, c = i % CH;
        constexpr int np = (SP - c * PB) < PB ? (SP - c * PB) : PB;
        const sptr_t src = (sptr_t)(xbase + (at + (uint32_t)r * row_bytes + (uint32_t)(c * PB) * kPixBytes));
        if constexpr (KH == 1) {
            sload_run<np * PD>(src, dst);   // the pixels of a batch are contiguous
        } else {
            // this wavefront's CW channel words of each pixel, CWT word pairs apart
#pragma unroll
            for (int j = 0; j < np; ++j) sload_run<PD>(src + j * (2 * CWT), dst + j * PD);
        }
    };

    int32_t acc[U];
    auto consume = [&](auto i_tag, const uint32_t* x) {
        constexpr int i = decltype(i_tag)::value;
        constexpr int r = i / CH, c = i % CH;
        constexpr int np = (SP - c * PB) < PB ? (SP - c * PB) : PB;
#pragma unroll
        for (int j = 0; j < np; ++j) {
            const int jj = c * PB + j;   // position in the strip
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int s = jj - u * ST;   // filter column of this pixel for output pixel u
                if (s < 0 || s >= R) continue;
#pragma unroll
                for (int cw = 0; cw < CW; ++cw) {
                    const plane2 ww = w[r * R + s][cw];
                    const uint32_t xh = x[j * PD + 2 * cw], xl = x[j * PD + 2 * cw + 1];
                    if (OP == OP_TERNARY) {
                        popc_acc(acc[u], (xh ^ ww.x) & ww.y);
                        popc_acc(acc[u], (xl ^ ww.x) & ww.y);
                    } else if (OP == OP_XOR_PAIR) {
                        popc_acc(acc[u], xh ^ ww.x);
                        popc_acc(acc[u], xl ^ ww.y);
                    } else {
                        popc_acc(acc[u], xh ^ ww.x);
                        popc_acc(acc[u], xh ^ ww.y);
                        popc_acc(acc[u], xl ^ ww.x);
                        popc_acc(acc[u], xl ^ ww.y);
                    }
                }
            }
        }
    };

    uint32_t buf[2][Sh::BUF];
    const uint32_t lane_out = (uint32_t)m;   // this lane's channel inside an output pixel
    const uint32_t lane_byte = lane_out * 4u;
    // raw buffer resources over the two outputs (the host guarantees they are below 4 GiB)
    constexpr int kRsrcFlags = 0x00020000;
    // cache policy of the output stores: device scope (sc1) + non-temporal (nt).  Measured: plain stores
    // 20.1 us on the 128-channel layer and 97 us on the 64 -> 256 1x1 layer, nt alone 19.2 / 84, sc1 alone
    // 18.3 / 81 but the kernel after it slows down, both together 18.3 / 84 with no such after-effect.
    constexpr int kStreamOut = 16 | 2;
    const __amdgpu_buffer_rsrc_t crsrc = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)p.out_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t frsrc = __builtin_amdgcn_make_buffer_rsrc(p.Cf, 0, (int)p.out_bytes, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t srsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.skip), 0, (int)p.out_bytes, kRsrcFlags);
    // Chaining epilogue: lane 2u+h stores half h (channels 32h..32h+31 of this wavefront's 64)
    // of output pixel u as one word pair of the next layer's input.
    const uint32_t xn_word = (uint32_t)(2 * mb + (lane & 1));
    const bool xn_lane_ok = lane < 2 * U && xn_word < (uint32_t)p.nCw;
    const uint32_t xn_lane_off = ((uint32_t)(lane >> 1) * (uint32_t)p.nCw + xn_word) * 8u;

    // One group: batch i+1 (or batch 0 of the next group) is in flight while batch i is
    // consumed.  A scalar-load wait waits for every outstanding load, so the wait for batch
    // i comes BEFORE batch i+1 is issued.  PAR = which buffer holds batch 0.
    auto run_group = [&](auto par_tag, int gi) {
        constexpr int PAR = decltype(par_tag)::value;
        // The SIMD's arbiter favours its oldest wavefront, so the wavefronts of a SIMD would finish
        // one after the other and the last would run its final groups alone, at half the issue rate.
        // A wavefront lowers its own priority as it nears its end: the ones behind catch up and all
        // finish together.
        {
            const int left = count - gi;   // groups still to do, this one included
            if (left >= 4) __builtin_amdgcn_s_setprio(3);
            else if (left == 3) __builtin_amdgcn_s_setprio(2);
            else if (left == 2) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        const uint32_t o0 = ooff, n0 = noff;
        const int nu = (wg == wgroups - 1) ? p.tailU : U;   // output pixels of this group that exist
        uint32_t goff_next = goff;
        if (kStrided) {
            if (gi + 1 < count) {
                const uint32_t g_keep = goff;
                wg += step_wg;
                const int c1 = wg >= wgroups ? 1 : 0;
                wg -= c1 ? wgroups : 0;
                ho += step_ho + c1;
                const int c2 = ho >= p.Ho ? 1 : 0;
                ho -= c2 ? p.Ho : 0;
                img += step_img + c2;
                locate();
                goff_next = goff;
                goff = g_keep;
            }
        } else if (gi + 1 < count) {
            if (wg + 1 < wgroups) {
                ++wg;
                goff_next = goff + kInStep;
                ooff += out_step;
                if (EPI == EPI_CHAIN) noff += nx_step;
            } else {
                wg = 0;
                ooff += out_tail;
                if (ho + 1 < p.Ho) {
                    ++ho;
                    goff_next = goff + in_row_adj;
                    if (EPI == EPI_CHAIN) noff += nx_row_adj;
                } else {
                    ho = 0;
                    goff_next = goff + in_img_adj;
                    if (EPI == EPI_CHAIN) noff += nx_img_adj;
                }
            }
        }
        // The skip values of the group are requested now and used after the K loop, where the
        // registers allow it; with eight resident channel words and seven accumulators they are
        // requested in the epilogue.
        constexpr bool kSkipEarly = !(CW >= 8 && U >= 7);
        float sk[U];
        auto load_skips = [&]() {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                sk[u] = neg0;
                if (p.skip != nullptr && u < nu)
                    sk[u] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(
                        srsrc, (int)lane_byte, (int)((o0 + (uint32_t)u * ldc) * 4u), 0));
            }
        };
        if constexpr (EPI == EPI_CHAIN && kSkipEarly) {
            if (kh == 0) load_skips();
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = 0;
        auto step = [&](auto i_tag) {
            constexpr int i = decltype(i_tag)::value;
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (i + 1 < NBATCH)
                issue(std::integral_constant<int, i + 1>{}, goff, buf[(PAR + i + 1) & 1]);
            else
                issue(std::integral_constant<int, 0>{}, goff_next, buf[(PAR + i + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            consume(i_tag, buf[(PAR + i) & 1]);
            __builtin_amdgcn_sched_barrier(0);
        };
        [&]<int... I>(std::integer_sequence<int, I...>) { (step(std::integral_constant<int, I>{}), ...); }
        (std::make_integer_sequence<int, NBATCH>{});
        goff = goff_next;
        if constexpr (KH > 1) {
            // Two slots per row block, alternating with the group: the barrier of group g+1 lies between
            // wavefront 0 reading slot (g & 1) and the others writing it again for group g+2.
            int32_t* const slot = handover + ((size_t)(mbl * 2 + (gi & 1)) * (KH - 1) * U) * 64 + lane;
            if (kh > 0) {
#pragma unroll
                for (int u = 0; u < U; ++u) slot[((kh - 1) * U + u) * 64] = acc[u];
            }
            __syncthreads();
            if (kh > 0) return;
#pragma unroll
            for (int h = 0; h < KH - 1; ++h)
#pragma unroll
                for (int u = 0; u < U; ++u) acc[u] += slot[(h * U + u) * 64];
        }
        asm volatile("" : "+v"(rc_raw));   // keeps the multiply below out of the prologue
        const int32_t rc = p.cmul * rc_raw;
        if constexpr (EPI == EPI_CHAIN) {
            // Layer chaining (Supplementary S1: batch norm folded into the layer, ReLU and the skip
            // connection fused, packing fused): the 64 channels of a wavefront are 64 lanes, so a
            // wave-wide ballot of the two quantizer comparisons IS the pair of plane words.
            if constexpr (!kSkipEarly) load_skips();
            uint32_t wx = 0, wy = 0;
            auto pixel = [&](auto u_tag) {
                constexpr int u = decltype(u_tag)::value;
                const int32_t v = (OP == OP_TERNARY) ? rc - acc[u] : (OP == OP_XOR_PAIR ? p.K - p.cmul * acc[u] : p.K - (acc[u] >> 1));
                float f = sc * (float)v;
                f = f + bs;
                f = f + sk[u];
                if (p.relu) {
                    // max(f, 0) that keeps a NaN a NaN (v_max_f32 alone would return the 0); the fp32
                    // output then shows the NaN, and the quantizer below gives it the value 0
                    f = (f < 0.0f) ? 0.0f : f;
                    asm volatile("" : "+v"(f));   // keeps this a scalar branch instead of a per-lane select
                }
                if (p.Cf != nullptr)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(f), frsrc, (int)lane_byte,
                                                          (int)((o0 + (uint32_t)u * ldc) * 4u), kStreamOut);
                // wave-wide comparisons; a NaN compares false and is given the value 0 (low plane bit nan_lo)
                uint64_t lo = __ballot(f >= p.t1);
                if (p.nan_lo != 0u) lo |= __ballot(f != f);
                lo &= ok_mask;
                const uint64_t hi = __ballot(f >= p.t2) & ok_mask;
                // lane 2u <- low halves, lane 2u+1 <- high halves of this pixel's ballots
                write_lane<2 * u>(wx, (uint32_t)hi);
                write_lane<2 * u + 1>(wx, (uint32_t)(hi >> 32));
                write_lane<2 * u>(wy, (uint32_t)lo);
                write_lane<2 * u + 1>(wy, (uint32_t)(lo >> 32));
            };
            [&]<int... UU>(std::integer_sequence<int, UU...>) {
                ((UU < nu ? (pixel(std::integral_constant<int, UU>{}), 0) : 0), ...);
            }(std::make_integer_sequence<int, U>{});
            if (xn_lane_ok && lane < 2 * nu) {
                plane2 word;
                word.x = wx;
                word.y = wy;
                *reinterpret_cast<plane2*>(reinterpret_cast<char*>(p.Xn) + (size_t)(n0 * 8u + xn_lane_off)) = word;
            }
        } else {
            // Outputs go through buffer resources: the address of a store is (resource base) + (lane's
            // channel, a constant VGPR) + (pixel offset, an SGPR), so no vector instruction computes
            // addresses.  They are written once and not read again by this kernel: streamed out.
            // Which outputs exist and whether the group is complete is decided once per group.
            auto emit = [&](auto has_c, auto has_f, auto full) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!decltype(full)::value && u >= nu) break;
                    const int32_t v = (OP == OP_TERNARY) ? rc - acc[u] : (OP == OP_XOR_PAIR ? p.K - p.cmul * acc[u] : p.K - (acc[u] >> 1));
                    const int soff = (int)((o0 + (uint32_t)u * ldc) * 4u);
                    if constexpr (decltype(has_c)::value)
                        __builtin_amdgcn_raw_buffer_store_b32((uint32_t)v, crsrc, (int)lane_byte, soff, kStreamOut);
                    if constexpr (decltype(has_f)::value) {
                        float f = sc * (float)v;
                        f = f + bs;
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(f), frsrc, (int)lane_byte, soff, kStreamOut);
                    }
                }
            };
            constexpr std::true_type yes{};
            constexpr std::false_type no{};
            const bool full = nu == U;
            if (p.C != nullptr && p.Cf != nullptr) {
                if (full) emit(yes, yes, yes); else emit(yes, yes, no);
            } else if (p.C != nullptr) {
                if (full) emit(yes, no, yes); else emit(yes, no, no);
            } else {
                if (full) emit(no, yes, yes); else emit(no, yes, no);
            }
        }
    };

    // this wavefront's channel words of every tap: weights into registers, activations by offset (xbase)
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int c = 0; c < CW; ++c) w[t][c] = wsrc[(int64_t)(t * CWT + kh * CW + c) * 64];
    seek();
    issue(std::integral_constant<int, 0>{}, goff, buf[0]);

    int gi = 0;
    while (gi < count) {
        run_group(std::integral_constant<int, 0>{}, gi);
        ++gi;
        if constexpr ((NBATCH & 1) != 0) {
            // an odd number of batches leaves the prefetched batch in the other buffer
            if (gi < count) {
                run_group(std::integral_constant<int, 1>{}, gi);
                ++gi;
            } else {
                break;
            }
        }
    }
}

// Wavefronts per SIMD that stay resident for a kernel at a workgroup size (asked once per
// instantiation and workgroup size; the answer depends on the register count the compiler reached).
// A workgroup has at most 16 wavefronts (four row blocks of up to four wavefronts each).  The slots are
// atomics: concurrent first calls compute the same value and store it twice, which is harmless.
constexpr int kMaxWavesPerGroup = 16;
struct OccupancyCache {
    std::atomic<int> slot[kMaxWavesPerGroup + 1];
};
template <typename Kernel>
int resident_waves_per_simd(Kernel kernel, int waves_per_group, size_t lds, OccupancyCache& cache) {
    if (waves_per_group < 1 || waves_per_group > kMaxWavesPerGroup) return 1;
    int v = cache.slot[waves_per_group].load(std::memory_order_relaxed);
    if (v == 0) {
        int nblk = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nblk, kernel, 64 * waves_per_group, lds) != hipSuccess ||
            nblk < 1)
            nblk = 1;
        const int waves = nblk * waves_per_group / 4;
        v = waves < 1 ? 1 : (waves > 8 ? 8 : waves);
        cache.slot[waves_per_group].store(v, std::memory_order_relaxed);
    }
    return v;
}

// Number of ranges of pixel groups (= wavefronts per block of 64 output channels).  All
// wavefronts are meant to be resident at once, the same number on every SIMD, and each
// should see enough groups to amortise loading its weights.  Tuning::stream_wps forces the
// wavefronts per SIMD (for measurements).
int plan_ranges(int64_t mblocks, int64_t ngroups, int occ) {
    // As many wavefronts per SIMD as stay resident, up to 6 (more only adds weight-load traffic at
    // the start); beyond four only while each still gets three pixel groups, and never more
    // wavefronts than groups.  (One or two wavefronts per SIMD issue the logic/popcount pairs at
    // 0.6x / 1.1x the nominal rate, four at 1.2x: small problems want the wavefronts, not the groups.)
    int64_t wps = occ < 6 ? occ : 6;
    while (wps > 4 && ngroups * mblocks < 3 * 1024 * wps) --wps;
    while (wps > 1 && ngroups * mblocks < 1024 * wps) --wps;
    const int forced = tuning().stream_wps;
    if (forced > 0) wps = forced < occ ? forced : occ;
    int64_t ranges = (1024 * wps) / mblocks;
    if (ranges < 1) ranges = 1;
    if (ranges > ngroups) ranges = ngroups;
    return (int)ranges;
}

template <int OP, int R, int CW, int CWT, int ST, int U>
int launch_inst(StreamParams p, int64_t out_rows, int64_t Wo, hipStream_t stream) {
    p.wgroups = (int32_t)((Wo + U - 1) / U);
    p.tailU = (int32_t)(Wo - (int64_t)(p.wgroups - 1) * U);
    const int64_t ngroups = out_rows * p.wgroups;
    if (ngroups <= 0 || ngroups > 0x7FFFFFF0LL) return -2;
    constexpr int KH = CWT / CW;                      // wavefronts per (row block, range)
    const int mblocks = (p.M + 63) / 64;
    // Row blocks per workgroup: four wavefronts per workgroup whatever KH is.  (With four row blocks of
    // four wavefronts each, a 512-channel workgroup filled a compute unit by itself, and the compute units
    // whose workgroup had one group more than the others' worked a third longer: 35.7 against 26.7 us.
    // Small workgroups let every compute unit hold some of both kinds.)
    const int wpb_max = KH >= 4 ? 1 : (KH == 2 ? 2 : 4);
    const int wpb = mblocks < wpb_max ? mblocks : wpb_max;
    const int waves = wpb * KH;
    static_assert(4 * KH <= kMaxWavesPerGroup, "occupancy cache too small for this workgroup");
    const size_t lds = KH > 1 ? (size_t)wpb * 2 * (KH - 1) * U * 64 * sizeof(int32_t) : 0;
    auto launch = [&](auto kernel, OccupancyCache& cache) {
        const int occ = resident_waves_per_simd(kernel, waves, lds, cache);
        const int ranges = plan_ranges((int64_t)mblocks * KH, ngroups, occ);
        p.gq = (int32_t)(ngroups / ranges);
        p.gr = (int32_t)(ngroups % ranges);
        dim3 grid((unsigned)(ranges * ((mblocks + wpb - 1) / wpb)));
        const LaunchTiming t = take_launch_timing();
        hipExtLaunchKernelGGL(kernel, grid, dim3(64 * waves), lds, stream, t.start, t.stop, 0, p);
        return hipGetLastError() == hipSuccess ? 0 : -1;
    };
    if (p.Xn != nullptr) {
        if constexpr (OP == OP_TERNARY) {
            static OccupancyCache cache{};
            return launch(stream_conv_kernel<OP, R, CW, CWT, ST, U, EPI_CHAIN>, cache);
        } else {
            return -3;
        }
    }
    static OccupancyCache cache{};
    return launch(stream_conv_kernel<OP, R, CW, CWT, ST, U, EPI_PLAIN>, cache);
}

// Output pixels per group for a filter size / channel-word count / stride.
constexpr int group_u(int R, int CW, int ST) {
    if (R == 3) return (ST == 1) ? (CW == 2 ? 8 : 4) : (CW >= 8 ? 2 : 4);
    return (CW >= 8) ? 4 : (CW == 4 ? 4 : 8);   // 1x1
}
// Channel words one wavefront keeps in registers.  3x3 filters over 512 channels do not fit one wavefront;
// over 256 channels they would, at three wavefronts per SIMD.  Both are split into wavefronts of four
// channel words (two per row block for 256 channels, four for 512), which leaves room for four or five
// wavefronts per SIMD: measured 10 % faster for 256 channels, and 6 % faster than eight-word pairs for 512.
constexpr int resident_cw(int R, int CWT, int ST, int U) {
    if (R != 3) return CWT;
    if (CWT >= 8) return 4;
    // 128 channels: pairs of two-word wavefronts pay with the seven-pixel groups and on the stride-2 layer
    // (chained trunk at batch 64: 31 -> 29.5 us, 20.9 -> 18.9 us); with groups of four at stride 1 (rows
    // that are no multiple of seven) the single four-word wavefront is faster, 17.9 against 19.3 us.
    // (Measured again with the priorities of today: one four-word wavefront with the seven-pixel groups takes
    // 17.2 against 15.0 us on the batch-32 layer and 15.5 against 13.9 us on the stride-2 layer.)
    if (CWT == 4 && (U == 7 || ST == 2)) return 2;
    return CWT;
}

// Second group size of a shape (0 = none).  ResNet's rows are 56, 28, 14 and 7 pixels wide: groups of
// seven leave no partly empty group at the end of a row.  (For 64-channel layers groups of fourteen
// were measured 3-5 % slower than the groups of eight, which already divide 56, and at stride 2
// groups of seven 10 % slower than groups of four.)
constexpr int alt_u(int R, int CW, int ST) {
    if (R != 3) return 0;
    if (ST == 2) return (CW == 4 || CW == 8) ? 7 : 0;
    return (CW == 4 || CW == 8 || CW == 16) ? 7 : 0;
}

// Output pixels per group for this call.  Tuning::u7_mode 0 switches the second group size off,
// 2 uses it wherever a kernel exists (for tests of those kernels on small inputs).
int pick_group_size(int op, int R, int Cw, int stride, int64_t out_rows, int64_t Wo, int64_t mblocks) {
    const int alt = alt_u(R, Cw, stride);
    if (alt != 0 && Wo % alt == 0) {
        const int mode = tuning().u7_mode;
        // 128 channels: always (with the two-word wavefront pairs that go with it, measured 15-20 % faster
        // from batch 2 to 32 at 28x28 and equal beyond); 256 and 512 channels: only where the larger groups
        // still leave every SIMD three of them (measured: slower at 1-2 per SIMD, faster from 3.5)
        const int64_t enough = Cw <= 4 ? 0 : 3 * 1024;
        if (mode == 2 || (mode != 0 && out_rows * (Wo / alt) * mblocks >= enough)) return alt;
    }
    return group_u(R, Cw, stride);
}

}  // namespace

bool stream_supported(int op, int R, int S, int Cw, int stride) {
    if (op != OP_TERNARY && op != OP_TWOBIT_TERNARY && op != OP_XOR_PAIR) return false;
    if (R != S || (stride != 1 && stride != 2)) return false;
    if (R == 3) return Cw == 2 || Cw == 4 || Cw == 8 || Cw == 16;
    if (R == 1) return Cw == 2 || Cw == 4 || Cw == 8 || Cw == 16;
    return false;
}

int launch_stream_conv(const StreamParams& p, int op, int R, int Cw, int stride, int64_t out_rows, int64_t Wo,
                       hipStream_t stream) {
    const int U = pick_group_size(op, R, Cw, stride, out_rows, Wo, (p.M + 63) / 64);
#define FATNN_STREAM_CASE(RR, CC, SS)                                                                          \
    if (R == RR && Cw == CC && stride == SS) {                                                                 \
        constexpr int UU = group_u(RR, CC, SS);                                                                \
        constexpr int RC = resident_cw(RR, CC, SS, UU);                                                        \
        if constexpr (alt_u(RR, CC, SS) != 0) {                                                                \
            constexpr int UA = alt_u(RR, CC, SS);                                                              \
            constexpr int RA = resident_cw(RR, CC, SS, UA);                                                    \
            if (U == UA) {                                                                                     \
                if (op == OP_TERNARY) return launch_inst<OP_TERNARY, RR, RA, CC, SS, UA>(p, out_rows, Wo, stream);   \
                if (op == OP_XOR_PAIR) return launch_inst<OP_XOR_PAIR, RR, RA, CC, SS, UA>(p, out_rows, Wo, stream); \
                return launch_inst<OP_TWOBIT_TERNARY, RR, RA, CC, SS, UA>(p, out_rows, Wo, stream);            \
            }                                                                                                  \
        }                                                                                                      \
        if (op == OP_TERNARY) return launch_inst<OP_TERNARY, RR, RC, CC, SS, UU>(p, out_rows, Wo, stream);    \
        if (op == OP_XOR_PAIR) return launch_inst<OP_XOR_PAIR, RR, RC, CC, SS, UU>(p, out_rows, Wo, stream);  \
        return launch_inst<OP_TWOBIT_TERNARY, RR, RC, CC, SS, UU>(p, out_rows, Wo, stream);                    \
    }
    FATNN_STREAM_CASE(3, 2, 1)
    FATNN_STREAM_CASE(3, 4, 1)
    FATNN_STREAM_CASE(3, 8, 1)
    FATNN_STREAM_CASE(3, 16, 1)
    FATNN_STREAM_CASE(3, 16, 2)
    FATNN_STREAM_CASE(3, 2, 2)
    FATNN_STREAM_CASE(3, 4, 2)
    FATNN_STREAM_CASE(3, 8, 2)
    FATNN_STREAM_CASE(1, 2, 1)
    FATNN_STREAM_CASE(1, 4, 1)
    FATNN_STREAM_CASE(1, 8, 1)
    FATNN_STREAM_CASE(1, 16, 1)
    FATNN_STREAM_CASE(1, 2, 2)
    FATNN_STREAM_CASE(1, 4, 2)
    FATNN_STREAM_CASE(1, 8, 2)
    FATNN_STREAM_CASE(1, 16, 2)
#undef FATNN_STREAM_CASE
    return -3;
}

}  // namespace fatnn
