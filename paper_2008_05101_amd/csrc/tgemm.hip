// Bit-plane GEMM / implicit-GEMM convolution kernels for gfx950.
//
// Ternary operator (Section 3.3).  With the activation codec bits x_hi, x_lo
// (Table 1, zero spelled 01), the weight sign bit s = (w == +1) and the weight
// non-zero bit nm = (w != 0) = complement of Eq. 6's mask, Eq. 7 splits into two
// bit-disjoint parts, mask & auxi and ~mask & xnor, so
//     popcount(TM) = #zero weights + 2 * #non-zero weights - P',
//     P' = popcount((x_hi ^ s) & nm) + popcount((x_lo ^ s) & nm),
// and Eq. 3 becomes  x . w = #non-zero weights - P'.  Everything that depends only
// on the weights is precomputed per row; the hot loop is one three-input logic
// operation (v_bitop3_b32) and one accumulating popcount (v_bcnt_u32_b32) per
// plane word: 2 + 2 VALU instructions per 32 elements.
//
// Two-bit operators (Eq. 2 with two planes per operand, Eq. 1 per plane pair):
// four xor and four popcounts per 32 elements, same tiling, for comparison.
//
// Tiling.  A workgroup of WM x WN wavefronts owns a (WM*8*TM) x (WN*8*TN) tile of
// the output.  A wavefront is an 8 x 8 grid of lanes, each lane holds TM x TN int32
// accumulators.  K is walked in steps of KT = 8 word pairs (256 elements): the
// packed tiles of both operands are staged global -> registers -> LDS (double
// buffered, one barrier per step) in [k-word][row] order, so that a lane's rows
// for one k-word are fetched with 128-bit LDS reads that are contiguous across the
// eight lanes of a group.
#include "fatnn_device.h"

#include <atomic>
#include <type_traits>

namespace fatnn {
namespace {

constexpr int KT = 8;        // k-words per LDS stage
constexpr int LDS_PAD = 4;   // plane2 elements of padding per k-word line (keeps 16 B alignment)

// acc += popcount(x) as the single instruction v_bcnt_u32_b32 (its second source is an
// addend).  Written as asm because the compiler otherwise re-associates a chain of
// such additions into popcounts with a zero addend plus a three-input add.
__device__ __forceinline__ void popc_acc(int32_t& acc, uint32_t x) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
}

template <int OP>
struct Acc;

template <>
struct Acc<OP_TERNARY> {
    static constexpr int kWords = 1;
    int32_t v;
    __device__ __forceinline__ int32_t& word(int) { return v; }
    __device__ __forceinline__ void clear() { v = 0; }
    __device__ __forceinline__ void step(plane2 w, plane2 a) {
        popc_acc(v, (a.x ^ w.x) & w.y);
        popc_acc(v, (a.y ^ w.x) & w.y);
    }
};

template <>
struct Acc<OP_TWOBIT_TERNARY> {
    static constexpr int kWords = 1;
    int32_t v;
    __device__ __forceinline__ int32_t& word(int) { return v; }
    __device__ __forceinline__ void clear() { v = 0; }
    __device__ __forceinline__ void step(plane2 w, plane2 a) {
        popc_acc(v, a.x ^ w.x);
        popc_acc(v, a.x ^ w.y);
        popc_acc(v, a.y ^ w.x);
        popc_acc(v, a.y ^ w.y);
    }
};

template <>
struct Acc<OP_TWOBIT_UNIFORM> {
    static constexpr int kWords = 3;
    int32_t s00, s01, s11;   // by weight of the plane pair: 1, 2, 4
    __device__ __forceinline__ int32_t& word(int i) { return i == 0 ? s00 : (i == 1 ? s01 : s11); }
    __device__ __forceinline__ void clear() { s00 = s01 = s11 = 0; }
    __device__ __forceinline__ void step(plane2 w, plane2 a) {
        popc_acc(s00, a.y ^ w.y);
        popc_acc(s01, a.x ^ w.y);
        popc_acc(s01, a.y ^ w.x);
        popc_acc(s11, a.x ^ w.x);
    }
};

// Plain xor-popcount over both words of a pair: the binary inner product of Eq. 1 (64 one-bit
// elements per pair), and the xnor rule of Eq. 4 without the zero-operand fix of Eq. 5-7.
template <>
struct Acc<OP_XOR_PAIR> {
    static constexpr int kWords = 1;
    int32_t v;
    __device__ __forceinline__ int32_t& word(int) { return v; }
    __device__ __forceinline__ void clear() { v = 0; }
    __device__ __forceinline__ void step(plane2 w, plane2 a) {
        popc_acc(v, a.x ^ w.x);
        popc_acc(v, a.y ^ w.y);
    }
};

template <int OP>
__device__ __forceinline__ int32_t finalize(const Acc<OP>& acc, const GemmParams& p, int32_t rowconst);

template <>
__device__ __forceinline__ int32_t finalize<OP_XOR_PAIR>(const Acc<OP_XOR_PAIR>& acc, const GemmParams& p, int32_t) {
    // binary (Eq. 1): 2 * popcount(xnor) - N = N - 2 * popcount(xor);  xnor rule on codecs: N - popcount(xor)
    return p.K - p.cmul * acc.v;
}

template <>
__device__ __forceinline__ int32_t finalize<OP_TERNARY>(const Acc<OP_TERNARY>& acc, const GemmParams&,
                                                        int32_t rowconst) {
    return rowconst - acc.v;
}
template <>
__device__ __forceinline__ int32_t finalize<OP_TWOBIT_TERNARY>(const Acc<OP_TWOBIT_TERNARY>& acc,
                                                               const GemmParams& p, int32_t) {
    // sum_mk (1/4) * (K - 2 * popcount(x_m ^ y_k))
    return p.K - (acc.v >> 1);
}
template <>
__device__ __forceinline__ int32_t finalize<OP_TWOBIT_UNIFORM>(const Acc<OP_TWOBIT_UNIFORM>& acc,
                                                               const GemmParams& p, int32_t) {
    // sum_mk 2^(m+k) * (K - 2 * popcount(x_m ^ y_k))
    return 9 * p.K - 2 * acc.s00 - 4 * acc.s01 - 8 * acc.s11;
}

// Even-share ("stream-K") schedule.  The work of a GEMM is cut into units of one K stage (KT k-words) of
// one output tile, numbered tile by tile; workgroup g of G owns the units [g*U/G, (g+1)*U/G), i.e. a run of
// whole tiles with possibly a piece of a tile at either end.  Every workgroup therefore does the same
// amount of arithmetic whatever the number of tiles is -- there is no last, partly filled round of tiles
// on the 256 compute units.  A piece hands its partial popcount sums over through `partial` (one slot per
// workgroup and end) and adds the number of its stages to the tile's counter; the piece whose addition
// completes the count collects the other slots and runs the epilogue, so nobody ever waits for anybody.
// The counters must be zero at launch and are zero again when the kernel has finished.
//
// Variant "whole tiles plus a split remainder" (whole > 0): the first `whole` workgroups take one whole tile
// each, as in the plain launch, and only the tiles that would form the last, partly filled round on the
// compute units are cut into even shares for the remaining workgroups, which are the first in dispatch
// order: a compute unit then runs q whole tiles and one piece instead of q or q + 1 tiles, and only the
// few split tiles pay for a hand-over.
struct StreamKArgs {
    int32_t* partial;    // [G - whole][2][tile accumulator words], written and read inside one launch
    int32_t* counters;   // [ntiles]
    int32_t nst;         // K stages per tile
    int32_t units;       // ntiles * nst
    int32_t whole;       // leading workgroups that own exactly one whole tile (0: even shares for all)
    // The shares without a division in the kernel: the first `extra` sharing workgroups own base + 1 units,
    // the others base; the two reciprocals only seed the search for the owner of a unit.
    int32_t base, extra;
    float inv_base1, inv_base;
};

// Fills in the share sizes for `groups` sharing workgroups (all of them, or those behind the whole tiles).
inline void set_shares(StreamKArgs& sk, int64_t groups) {
    const int64_t shared_units = (int64_t)sk.units - (int64_t)sk.whole * sk.nst;
    sk.base = (int32_t)(shared_units / groups);
    sk.extra = (int32_t)(shared_units % groups);
    sk.inv_base1 = 1.0f / (float)(sk.base + 1);
    sk.inv_base = sk.base > 0 ? 1.0f / (float)sk.base : 0.0f;
}

template <int OP, int WM, int WN, int TM, int TN, bool CONV, bool STREAMK>
__global__ __launch_bounds__(64 * WM * WN, (TM * TN <= 4 ? 8 : 2)) void plane_gemm_kernel(const GemmParams p, const int tiles_m,
                                                                        const int ntiles, const StreamKArgs sk) {
    constexpr int NT = 64 * WM * WN;
    constexpr int BM = WM * 8 * TM;
    constexpr int BN = WN * 8 * TN;
    constexpr int LW = (BM * KT) / NT;   // staged word pairs per thread, weights
    constexpr int LA = (BN * KT) / NT;   // ... activations
    static_assert((BM * KT) % NT == 0 && (BN * KT) % NT == 0, "tile does not divide over the threads");
    static_assert(TM % 2 == 0 && TN % 2 == 0, "lanes own row pairs");
    static_assert(NT % KT == 0, "a thread keeps one k-word slot");
    static_assert(!(STREAMK && CONV), "the even-share schedule is built for the GEMM addressing only");
    constexpr int ROWS_PER_PASS = NT / KT;
    constexpr int PW = BM + LDS_PAD;
    constexpr int PA = BN + LDS_PAD;

    __shared__ __attribute__((aligned(16))) plane2 Ws[2][KT][PW];
    __shared__ __attribute__((aligned(16))) plane2 As[2][KT][PA];
    __shared__ int32_t ticket;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
    // logical indices (gridDim.x is a multiple of 8).
    // (With a split remainder the piece workgroups come first in dispatch order -- they are then resident
    // from the start whatever the occupancy -- and take the logical indices behind the whole tiles; the
    // runs per XCD are formed over the whole-tile workgroups, whose number is a multiple of 8 as well.)
    int logical;
    if (STREAMK && sk.whole > 0) {
        const int pieces = (int)gridDim.x - sk.whole;
        const int b = (int)blockIdx.x - pieces;
        logical = b < 0 ? sk.whole + (int)blockIdx.x : (b & 7) * (sk.whole >> 3) + (b >> 3);
    } else {
        logical = (int)(blockIdx.x & 7) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3);
    }
    if (!STREAMK && logical >= ntiles) return;
    const int tiles_n = ntiles / tiles_m;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave % WM;
    const int wave_n = wave / WM;
    const int ly = lane >> 3;
    const int lx = lane & 7;

    const int ld_j = tid % KT;
    const int ld_r = tid / KT;

    // Lane-owned rows/columns inside the wavefront tile: pairs at a stride of 16, so
    // that one 128-bit LDS read is contiguous over the eight lane groups.
    const int wrow = wave_m * 8 * TM + ly * 2;
    const int wcol = wave_n * 8 * TN + lx * 2;

    Acc<OP> acc[TM][TN];
    int row0 = 0, col0 = 0;
    // The SIMD's arbiter favours its oldest wavefront: of the workgroups that share a compute unit the
    // first would run ahead and finish early, and the last would do its final stages alone, when a SIMD
    // issues at half its rate (measured: four equal workgroups per compute unit finished at 17, 24, 31 and
    // 38 us).  Every wavefront therefore lowers its own priority as its share of the work proceeds (four
    // levels), which keeps the workgroups of a compute unit within a quarter of their work of each other.
    // (Not for the 128 x 128 tile: its workgroups come in several rounds per compute unit, and 4096^3 was
    // measured 3.6 % slower with it.)
    constexpr bool kPaced = TM * TN <= 16;
    // (work_mark[k] = the first stage at which k quarters of the work are done: the four levels without a
    // division per stage)
    int work_done = 0, work_mark[3] = {1, 1, 1};
    auto set_work = [&](int total) {
#pragma unroll
        for (int k = 0; k < 3; ++k) work_mark[k] = ((k + 1) * total + 3) >> 2;
    };
    auto pace = [&]() {
        if constexpr (!kPaced) return;
        if (work_done < work_mark[0]) __builtin_amdgcn_s_setprio(3);
        else if (work_done < work_mark[1]) __builtin_amdgcn_s_setprio(2);
        else if (work_done < work_mark[2]) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
        ++work_done;
    };

    // Logical tiles are ordered in bands of kBand tile rows walked column by column, so that the
    // ~64 tiles resident on one XCD at a time form a roughly square block (8 weight panels x 8
    // activation panels) and share their operand panels in that XCD's L2.
    auto locate_tile = [&](int t) {
        constexpr int kBand = 8;
        const int band = t / (kBand * tiles_n);
        const int band_m0 = band * kBand;
        const int band_rows = (tiles_m - band_m0) < kBand ? (tiles_m - band_m0) : kBand;
        const int in_band = t - band * kBand * tiles_n;
        row0 = (band_m0 + in_band % band_rows) * BM;
        col0 = (in_band / band_rows) * BN;
    };

    // Accumulates the K stages [kt0, kt1) of the tile at (row0, col0) into acc (cleared first).
    auto run_stages = [&](const int kt0, const int kt1) {
        // ---- global addressing of the staged loads ------------------------------------------
        // Both operands are read through buffer resources: a load whose byte offset is at or
        // beyond num_records returns zero, which takes care of rows past M / N without any
        // branch; k-words past the end of a row are sent to kOutOfRange on purpose.
        constexpr uint32_t kOutOfRange = 0x80000000u;
        constexpr int kRsrcFlags = 0x00020000;   // raw buffer, 32-bit data format
        const int64_t wbase = (int64_t)row0 * p.Kw;
        const int64_t wleft = ((int64_t)p.M * p.Kw - wbase) * (int64_t)sizeof(plane2);
        const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<plane2*>(p.W + wbase), 0, (int)(wleft < 0x7FFFFFFFLL ? wleft : 0x7FFFFFFFLL), kRsrcFlags);
        uint32_t woff[LW];
#pragma unroll
        for (int i = 0; i < LW; ++i) woff[i] = (uint32_t)(ld_r + i * ROWS_PER_PASS) * (uint32_t)p.Kw * 8u;

        int64_t abase, aleft;
        uint32_t aoff[LA];   // GEMM: byte offset of the row.  conv: byte offset of the column's image
        int hi0[LA], wi0[LA];
        if (CONV) {
            const int64_t img = (int64_t)p.H * p.Wd * p.Cw;          // word pairs per image
            const int b0 = col0 / (p.Ho * p.Wo);
            abase = (int64_t)b0 * img;
            aleft = ((int64_t)p.B * img - abase) * (int64_t)sizeof(plane2);
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                const int n = col0 + ld_r + i * ROWS_PER_PASS;
                const int nn = n < p.N ? n : col0;   // columns past N are never stored; keep them in range
                const int wo = nn % p.Wo;
                const int t = nn / p.Wo;
                const int ho = t % p.Ho;
                const int b = t / p.Ho;
                hi0[i] = ho * p.stride - p.pad;
                wi0[i] = wo * p.stride - p.pad;
                aoff[i] = (uint32_t)(b - b0) * (uint32_t)img * 8u;
            }
        } else {
            abase = (int64_t)col0 * p.Kw;
            aleft = ((int64_t)p.N * p.Kw - abase) * (int64_t)sizeof(plane2);
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                hi0[i] = wi0[i] = 0;
                aoff[i] = (uint32_t)(ld_r + i * ROWS_PER_PASS) * (uint32_t)p.Kw * 8u;
            }
        }
        const __amdgpu_buffer_rsrc_t arsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<plane2*>(p.A + abase), 0, (int)(aleft < 0x7FFFFFFFLL ? aleft : 0x7FFFFFFFLL), kRsrcFlags);

        auto load2 = [](const __amdgpu_buffer_rsrc_t& r, uint32_t off) {
            const auto v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
            plane2 o;
            o.x = v[0];
            o.y = v[1];
            return o;
        };

        // Small tiles finish a stage faster than a global load returns, so they keep two stages in
        // flight (two register sets); the large tiles have no registers to spare for that.
        constexpr bool kTwoAhead = (LW + LA) <= 4;
        constexpr int NSETS = kTwoAhead ? 2 : 1;
        plane2 wregs[NSETS][LW], aregs[NSETS][LA];
        auto fetch = [&](int kt, auto set_tag) {
            constexpr int set = decltype(set_tag)::value;
            plane2(&wreg)[LW] = wregs[set];
            plane2(&areg)[LA] = aregs[set];
            const int kw = kt * KT + ld_j;
            const bool kok = kw < p.Kw;
#pragma unroll
            for (int i = 0; i < LW; ++i) wreg[i] = load2(wrsrc, kok ? woff[i] + (uint32_t)kw * 8u : kOutOfRange);
            if (CONV) {
                // k-word -> (filter tap, channel word); c is innermost in K.  No integer division: the
                // channel-word count of the usual layers is a power of two, and a tap index below nine
                // splits into row and column of a 3 x 3 filter with one multiply (S is 1 or 3).
                const int kwc = kok ? kw : 0;
                const int tap = p.cw_shift >= 0 ? (kwc >> p.cw_shift) : kwc / p.Cw;
                const int cw = kwc - tap * p.Cw;
                const int r = p.S == 1 ? tap : (tap * 11) >> 5;
                const int s = tap - r * p.S;
#pragma unroll
                for (int i = 0; i < LA; ++i) {
                    const int hi = hi0[i] + r;
                    const int wi = wi0[i] + s;
                    const bool inside = (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.Wd;
                    const uint32_t off = aoff[i] + (uint32_t)((hi * p.Wd + wi) * p.Cw + cw) * 8u;
                    plane2 v = load2(arsrc, (kok && inside) ? off : kOutOfRange);
                    // a padded tap is the value 0; only its low plane can be non-zero (codec 01)
                    v.y |= (kok && !inside) ? p.pad_y : 0u;
                    areg[i] = v;
                }
            } else {
#pragma unroll
                for (int i = 0; i < LA; ++i) areg[i] = load2(arsrc, kok ? aoff[i] + (uint32_t)kw * 8u : kOutOfRange);
            }
        };
        auto stage = [&](int buf, auto set_tag) {
            constexpr int set = decltype(set_tag)::value;
#pragma unroll
            for (int i = 0; i < LW; ++i) Ws[buf][ld_j][ld_r + i * ROWS_PER_PASS] = wregs[set][i];
#pragma unroll
            for (int i = 0; i < LA; ++i) As[buf][ld_j][ld_r + i * ROWS_PER_PASS] = aregs[set][i];
        };
        constexpr std::integral_constant<int, 0> set0{};
        constexpr std::integral_constant<int, NSETS - 1> set1{};

#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int c = 0; c < TN; ++c) acc[i][c].clear();

        auto read_frag = [&](int buf, int j, plane2 (&w)[TM], plane2 (&a)[TN]) {
#pragma unroll
            for (int q = 0; q < TM / 2; ++q) {
                const uint4 v = *reinterpret_cast<const uint4*>(&Ws[buf][j][wrow + q * 16]);
                w[2 * q].x = v.x; w[2 * q].y = v.y;
                w[2 * q + 1].x = v.z; w[2 * q + 1].y = v.w;
            }
#pragma unroll
            for (int q = 0; q < TN / 2; ++q) {
                const uint4 v = *reinterpret_cast<const uint4*>(&As[buf][j][wcol + q * 16]);
                a[2 * q].x = v.x; a[2 * q].y = v.y;
                a[2 * q + 1].x = v.z; a[2 * q + 1].y = v.w;
            }
        };

        // One stage of the K loop from LDS buffer buf.  Fragments of k-word j+1 are read from LDS
        // while k-word j is consumed.  The scheduling fences keep the compiler from hoisting every
        // LDS read of the stage to its top (which needs more registers than there are).
        auto compute_words = [&](int buf, int jn, auto full_tag) {
            constexpr bool kFull = decltype(full_tag)::value;   // all KT k-words exist: no per-word test
            plane2 w[2][TM], a[2][TN];
            read_frag(buf, 0, w[0], a[0]);
#pragma unroll
            for (int j = 0; j < KT; ++j) {
                if (!kFull && j >= jn) break;
                if (j + 1 < KT && (kFull || j + 1 < jn)) read_frag(buf, j + 1, w[(j + 1) & 1], a[(j + 1) & 1]);
                FATNN_VOP3_RUN_PHASE();
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int c = 0; c < TN; ++c) acc[i][c].step(w[j & 1][i], a[j & 1][c]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        auto compute = [&](int kt, int buf) {
            // jn = k-words of this stage that exist (all KT except in the last, partial stage); the per-word
            // test is a scalar branch.  With the 32 x 32 tile a k-word is only sixteen vector instructions, and
            // two scalar tests per k-word weigh on it: its full stages run a copy without the tests (512 x N x K
            // with 1 / 4 / 6 / 8 tiles per compute unit: K = 4608 19.5 -> 13.2, 24.0 -> 20.4, 30.1 -> 27.8,
            // 38.1 -> 39.4 us; K = 2304 11.4 -> 8.2, 13.7 -> 12.1, 17.2 -> 18.1, 22.9 -> 22.0 us).  The same
            // copy for the 64 x 64 tile lets the compiler hoist LDS reads (108 instead of 76 registers, four
            // instead of six wavefronts per SIMD); reading fragments two k-words ahead changes nothing.  The
            // convolution front end keeps the tests: its three bench layers read 24.1 / 41.4 / 40.0 us with the
            // copy against 25.0 / 42.1 / 37.0 us without.
            const int jn = p.Kw - kt * KT;
            if constexpr (TM * TN <= 4 && !CONV) {
                if (jn >= KT) {
                    compute_words(buf, KT, std::true_type{});
                    return;
                }
            }
            compute_words(buf, jn, std::false_type{});
        };
        if constexpr (!kTwoAhead) {
            fetch(kt0, set0);
            stage(0, set0);
            __syncthreads();
            for (int kt = kt0; kt < kt1; ++kt) {
                const int buf = (kt - kt0) & 1;
                pace();
                if (kt + 1 < kt1) fetch(kt + 1, set0);
                compute(kt, buf);
                if (kt + 1 < kt1) stage(buf ^ 1, set0);
                __syncthreads();
            }
        } else {
            // stage kt+1 waits in one register set while stage kt+2 is being loaded into the other
            fetch(kt0, set0);
            if (kt0 + 1 < kt1) fetch(kt0 + 1, set1);
            stage(0, set0);
            __syncthreads();
            for (int kt = kt0; kt < kt1; kt += 2) {
                pace();
                if (kt + 2 < kt1) fetch(kt + 2, set0);
                compute(kt, 0);
                if (kt + 1 < kt1) stage(1, set1);
                __syncthreads();
                if (kt + 1 >= kt1) break;
                pace();
                if (kt + 3 < kt1) fetch(kt + 3, set1);
                compute(kt + 1, 1);
                if (kt + 2 < kt1) stage(0, set0);
                __syncthreads();
            }
        }
    };

    // ---- epilogue: Eq. 3's subtraction, then the optional fp32 scale -----------------------
    auto epilogue = [&]() {
    // (column n = col0 + wcol + ... is even, so a pair is 8-byte aligned when the row pitch and the base are)
    const bool pair_c = p.ldc_n == 1 && (p.ldc_m & 1) == 0 && (reinterpret_cast<uintptr_t>(p.C) & 7) == 0;
    const bool pair_f = p.ldf_n == 1 && (p.ldf_m & 1) == 0 && (reinterpret_cast<uintptr_t>(p.Cf) & 7) == 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = row0 + wrow + (i >> 1) * 16 + (i & 1);
        if (m >= p.M) continue;
        int32_t rc = 0;
        if (OP == OP_TERNARY) rc = p.cmul * p.rowc[m];
        float sc = 0.f, bs = 0.f;
        if (p.Cf != nullptr) {
            sc = p.scale[m];
            if (p.bias != nullptr) bs = p.bias[m];
        }
        // A lane's columns come in adjacent pairs (c, c+1): where the output is column-contiguous and
        // 8-byte aligned the pair is one 64-bit store.  (Plain stores: a wavefront writes 64-byte pieces of
        // rows, which L2 merges with the neighbouring wavefront's; non-temporal stores were 10-15 % slower.)
#pragma unroll
        for (int c = 0; c < TN; c += 2) {
            const int n = col0 + wcol + (c >> 1) * 16;
            if (n >= p.N) continue;
            const int32_t v0 = finalize<OP>(acc[i][c], p, rc);
            const int32_t v1 = finalize<OP>(acc[i][c + 1], p, rc);
            const bool two = n + 1 < p.N;
            if (p.C != nullptr) {
                int32_t* dst = p.C + ((int64_t)m * p.ldc_m + (int64_t)n * p.ldc_n);
                if (pair_c && two) {
                    typedef int32_t i32x2 __attribute__((ext_vector_type(2)));
                    const i32x2 v = {v0, v1};
                    *reinterpret_cast<i32x2*>(dst) = v;
                } else {
                    dst[0] = v0;
                    if (two) dst[p.ldc_n] = v1;
                }
            }
            if (p.Cf != nullptr) {
                float f0 = __fmul_rn(sc, (float)v0), f1 = __fmul_rn(sc, (float)v1);
                if (p.bias != nullptr) {
                    f0 = __fadd_rn(f0, bs);
                    f1 = __fadd_rn(f1, bs);
                }
                float* dst = p.Cf + ((int64_t)m * p.ldf_m + (int64_t)n * p.ldf_n);
                if (pair_f && two) {
                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                    const f32x2 v = {f0, f1};
                    *reinterpret_cast<f32x2*>(dst) = v;
                } else {
                    dst[0] = f0;
                    if (two) dst[p.ldf_n] = f1;
                }
            }
        }
    }
    };

    const int nkt = (p.Kw + KT - 1) / KT;
    if constexpr (!STREAMK) {
        set_work(nkt);
        locate_tile(logical);
        run_stages(0, nkt);
        epilogue();
    } else {
        if (sk.whole > 0 && logical < sk.whole) {
            // a whole tile of a split-remainder launch: the plain path, kept apart from the bookkeeping of
            // the pieces below so that it runs with the plain kernel's registers
            set_work(nkt);
            locate_tile(logical);
            run_stages(0, nkt);
            epilogue();
            return;
        }
        constexpr int kTileWords = TM * TN * Acc<OP>::kWords * NT;   // accumulator words of a tile
        const int G = (int)gridDim.x;
        const int nst = sk.nst;
        // first unit of workgroup g: one tile each up to `whole`, even shares of the rest beyond it
        // (all in 32 bits: the host keeps the number of units below 2^31)
        const int whole = sk.whole;
        const int whole_units = whole * nst;
        auto first_unit = [&](int g) {
            const int i = g - whole;
            return g <= whole ? g * nst : whole_units + i * sk.base + (i < sk.extra ? i : sk.extra);
        };
        const int u_begin = first_unit(logical), u_end = first_unit(logical + 1);
        if (u_begin >= u_end) return;
        set_work(u_end - u_begin);
        const int tile_first = u_begin / nst, tile_last = (u_end - 1) / nst;
        const int nseg = tile_last - tile_first + 1;
        // The piece at the end of the range (the tile is finished by the next workgroup) is done first:
        // both halves of a shared tile are then ready early in the life of their workgroups, and the
        // hand-over is hidden behind the whole tiles that follow instead of sitting at the kernel's end.
        const bool tail_piece = u_end < (tile_last + 1) * nst;
        for (int idx = 0; idx < nseg; ++idx) {
            const int j = (tail_piece && nseg > 1) ? (idx == 0 ? nseg - 1 : idx - 1) : idx;
            const int tile = tile_first + j;
            const int t_begin = tile * nst;
            const int s0 = (u_begin > t_begin ? u_begin : t_begin) - t_begin;
            const int s1 = (u_end < t_begin + nst ? u_end : t_begin + nst) - t_begin;
            locate_tile(tile);
            run_stages(s0, s1);
            if (s0 == 0 && s1 == nst) {
                epilogue();
                continue;
            }
            // A piece of a shared tile.  Its partial popcount sums go to this workgroup's slot (slot 0 = a
            // piece that continues a tile, slot 1 = a piece that begins one) as device-scope atomic stores,
            // which write through to the level all XCDs share; the wait below returns when every one of them
            // has been acknowledged, and only then, after the workgroup's barrier, are the piece's stages
            // added to the tile's count.  The piece that completes the count reads the other slots with
            // device-scope atomic loads (which never take a stale line from the XCD's own L2), adds them to
            // the sums it still holds in registers, and runs the epilogue.  No cache is written back or
            // invalidated: a release / acquire fence pair around plain stores flushes or drops the XCD's
            // whole L2, operands included, and was measured four times slower than the plain kernel; adding
            // all pieces into one slot with atomic read-modify-writes suffered from their contention.
            int32_t* const mine = sk.partial + (int64_t)((logical - whole) * 2 + (s0 == 0 ? 1 : 0)) * kTileWords + tid;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int c = 0; c < TN; ++c)
#pragma unroll
                    for (int q = 0; q < Acc<OP>::kWords; ++q)
                        __hip_atomic_store(mine + ((i * TN + c) * Acc<OP>::kWords + q) * NT, acc[i][c].word(q),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the stores above have completed
            __syncthreads();
            if (tid == 0)
                ticket = __hip_atomic_fetch_add(sk.counters + tile, s1 - s0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const bool last = ticket + (s1 - s0) == nst;
            __syncthreads();   // everybody has read the ticket before a later piece overwrites it
            if (!last) continue;
            // leave the counter at zero for the next launch
            if (tid == 0) __hip_atomic_store(sk.counters + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // the other pieces of this tile: every workgroup whose range meets [t_begin, t_begin + nst)
            // (the reciprocals give the owner of the tile's first unit to within a few; the two loops settle it)
            const int u_rel = t_begin - whole_units, knee = sk.extra * (sk.base + 1);
            int g = u_rel < knee ? (int)((float)u_rel * sk.inv_base1)
                                 : sk.extra + (int)((float)(u_rel - knee) * sk.inv_base);
            g = whole + (g < 0 ? 0 : (g > G - whole - 1 ? G - whole - 1 : g));
            while (g > whole && first_unit(g) > t_begin) --g;
            while (first_unit(g + 1) <= t_begin) ++g;
            for (; g < G && first_unit(g) < t_begin + nst; ++g) {
                if (g == logical) continue;
                if (first_unit(g + 1) <= first_unit(g)) continue;   // a workgroup without units
                const int slot = first_unit(g) > t_begin ? 0 : 1;
                const int32_t* const theirs = sk.partial + (int64_t)((g - whole) * 2 + slot) * kTileWords + tid;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int c = 0; c < TN; ++c)
#pragma unroll
                        for (int q = 0; q < Acc<OP>::kWords; ++q)
                            acc[i][c].word(q) += __hip_atomic_load(theirs + ((i * TN + c) * Acc<OP>::kWords + q) * NT,
                                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            epilogue();
        }
    }
}

int compute_units();

// ---- few columns, long K: fully connected layers at batch 17-128 -------------------------------------
// Supplementary S1 treats a fully connected layer as a convolution whose filter covers the whole feature
// map: a GEMM with few columns (the batch) and a long K.  Its output has too few tiles to fill the chip and
// each tile's K loop is a chain of load latencies, so here the K range of a BM x 32 output tile is split
// over the eight wavefronts of a workgroup.  Every wavefront computes the whole tile over its eighth of K
// (8 x 8 lanes, TM x 4 accumulators per lane) from operands it stages itself in a private part of LDS --
// no barrier inside the K loop, the wavefronts run freely -- and the eight partial popcount sums of Eq. 3
// meet in LDS once, at the end, where each thread finishes two neighbouring outputs.
constexpr int DK_WAVES = 8;       // wavefronts per workgroup = parts of K
constexpr int DK_KC = 8;          // k-words staged per chunk
constexpr int DK_BN = 32;         // columns per tile

template <int OP, int TM>
__global__ __launch_bounds__(64 * DK_WAVES) void deepk_gemm_kernel(const GemmParams p, const int tiles_m) {
    constexpr int TN = 4, BM = 8 * TM, BN = DK_BN;
    constexpr int PW = BM + LDS_PAD, PA = BN + LDS_PAD;
    constexpr int kAccWords = TM * TN * Acc<OP>::kWords;
    constexpr int kStageBytes = DK_KC * (PW + PA) * (int)sizeof(plane2);   // per wavefront
    constexpr int kReduceBytes = kAccWords * 64 * 4;                       // per wavefront
    constexpr int kWaveBytes = kStageBytes > kReduceBytes ? kStageBytes : kReduceBytes;
    __shared__ __attribute__((aligned(16))) char lds[DK_WAVES * kWaveBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ly = lane >> 3, lx = lane & 7;
    const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    plane2(*Ws)[PW] = reinterpret_cast<plane2(*)[PW]>(lds + wave * kWaveBytes);
    plane2(*As)[PA] = reinterpret_cast<plane2(*)[PA]>(lds + wave * kWaveBytes + DK_KC * PW * (int)sizeof(plane2));

    // this wavefront's part of K, cut into equal chunks of at most DK_KC k-words
    const int per_wave = (p.Kw + DK_WAVES - 1) / DK_WAVES;
    const int kb = wave * per_wave;
    const int ke = (kb + per_wave < p.Kw) ? kb + per_wave : p.Kw;
    const int nchunks = (per_wave + DK_KC - 1) / DK_KC;
    const int kc = (per_wave + nchunks - 1) / nchunks;

    // Staging: a lane fetches two neighbouring k-words of one row per pass, four lanes cover a row's
    // DK_KC k-words (64 contiguous bytes), a pass covers sixteen rows.  Buffer loads: offsets at or beyond
    // num_records return zero, which serves rows past M / N; k-words outside [k0, k1) are sent there.
    // Two chunks are in flight (two register sets): the first wait pays the memory latency for both.
    constexpr uint32_t kOutOfRange = 0x80000000u;
    constexpr int kRsrcFlags = 0x00020000;
    constexpr int WPASS = BM / 16, APASS = BN / 16;
    const int64_t wbase = (int64_t)row0 * p.Kw, abase = (int64_t)col0 * p.Kw;
    const int64_t wleft = ((int64_t)p.M * p.Kw - wbase) * 8, aleft = ((int64_t)p.N * p.Kw - abase) * 8;
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<plane2*>(p.W + wbase), 0, (int)(wleft < 0x7FFFFFFFLL ? wleft : 0x7FFFFFFFLL), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t arsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<plane2*>(p.A + abase), 0, (int)(aleft < 0x7FFFFFFFLL ? aleft : 0x7FFFFFFFLL), kRsrcFlags);
    const int st_row = lane >> 2, st_kp = (lane & 3) * 2;
    auto load2 = [](const __amdgpu_buffer_rsrc_t& r, uint32_t off) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
        plane2 o;
        o.x = v[0];
        o.y = v[1];
        return o;
    };
    plane2 wreg[2][WPASS][2], areg[2][APASS][2];
    auto fetch = [&](int k0, auto set_tag) {
        constexpr int set = decltype(set_tag)::value;
        const int k1 = (k0 + kc < ke) ? k0 + kc : ke;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int kw = k0 + st_kp + h;
            const bool ok = kw < k1;
#pragma unroll
            for (int i = 0; i < WPASS; ++i)
                wreg[set][i][h] =
                    load2(wrsrc, ok ? ((uint32_t)(st_row + 16 * i) * (uint32_t)p.Kw + (uint32_t)kw) * 8u : kOutOfRange);
#pragma unroll
            for (int i = 0; i < APASS; ++i)
                areg[set][i][h] =
                    load2(arsrc, ok ? ((uint32_t)(st_row + 16 * i) * (uint32_t)p.Kw + (uint32_t)kw) * 8u : kOutOfRange);
        }
    };
    auto stage = [&](auto set_tag) {
        constexpr int set = decltype(set_tag)::value;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int i = 0; i < WPASS; ++i) Ws[st_kp + h][st_row + 16 * i] = wreg[set][i][h];
#pragma unroll
            for (int i = 0; i < APASS; ++i) As[st_kp + h][st_row + 16 * i] = areg[set][i][h];
        }
    };
    constexpr std::integral_constant<int, 0> set0{};
    constexpr std::integral_constant<int, 1> set1{};

    Acc<OP> acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int c = 0; c < TN; ++c) acc[i][c].clear();
    const int wrow = ly * 2, wcol = lx * 2;
    auto read_frag = [&](int j, plane2 (&w)[TM], plane2 (&a)[TN]) {
#pragma unroll
        for (int q = 0; q < TM / 2; ++q) {
            const uint4 v = *reinterpret_cast<const uint4*>(&Ws[j][wrow + q * 16]);
            w[2 * q].x = v.x; w[2 * q].y = v.y;
            w[2 * q + 1].x = v.z; w[2 * q + 1].y = v.w;
        }
#pragma unroll
        for (int q = 0; q < TN / 2; ++q) {
            const uint4 v = *reinterpret_cast<const uint4*>(&As[j][wcol + q * 16]);
            a[2 * q].x = v.x; a[2 * q].y = v.y;
            a[2 * q + 1].x = v.z; a[2 * q + 1].y = v.w;
        }
    };
    // LDS operations of one wavefront execute in the order they are issued; the fences only keep the
    // compiler from moving the reads of a chunk above the writes that fill it (other lanes' writes).
    auto wave_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    auto compute = [&](int k0) {
        const int jn = (k0 + kc < ke ? kc : ke - k0);
        plane2 w[2][TM], a[2][TN];
        read_frag(0, w[0], a[0]);
#pragma unroll
        for (int j = 0; j < DK_KC; ++j) {
            if (j < jn) {   // wave-uniform
                if (j + 1 < DK_KC && j + 1 < jn) read_frag(j + 1, w[(j + 1) & 1], a[(j + 1) & 1]);
                FATNN_VOP3_RUN_PHASE();
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int c = 0; c < TN; ++c) acc[i][c].step(w[j & 1][i], a[j & 1][c]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    if (kb < ke) {
        fetch(kb, set0);
        if (kb + kc < ke) fetch(kb + kc, set1);
        for (int k0 = kb; k0 < ke; k0 += 2 * kc) {
            wave_sync();                                  // the previous chunk has been read
            stage(set0);
            if (k0 + 2 * kc < ke) fetch(k0 + 2 * kc, set0);   // in flight while two chunks are consumed
            wave_sync();
            compute(k0);
            if (k0 + kc >= ke) break;
            wave_sync();
            stage(set1);
            if (k0 + 3 * kc < ke) fetch(k0 + 3 * kc, set1);
            wave_sync();
            compute(k0 + kc);
        }
    }

    // ---- the eight partial sums meet: [wavefront][accumulator word][lane] --------------------------------
    __syncthreads();   // every wavefront is done with its staging area (the sums reuse the space)
    int32_t* const red = reinterpret_cast<int32_t*>(lds);
    constexpr int kWaveWords = kWaveBytes / 4;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
            for (int q = 0; q < Acc<OP>::kWords; ++q)
                red[wave * kWaveWords + ((i * TN + c) * Acc<OP>::kWords + q) * 64 + lane] = acc[i][c].word(q);
    __syncthreads();
    // thread (wave, lane) finishes the accumulator pairs wave, wave + 8, ... of `lane`: outputs (m, n), (m, n + 1)
    constexpr int kPairs = TM * TN / 2;
    constexpr int kRounds = (kPairs + DK_WAVES - 1) / DK_WAVES;
    const bool pair_c = p.ldc_n == 1 && (p.ldc_m & 1) == 0 && (reinterpret_cast<uintptr_t>(p.C) & 7) == 0;
    const bool pair_f = p.ldf_n == 1 && (p.ldf_m & 1) == 0 && (reinterpret_cast<uintptr_t>(p.Cf) & 7) == 0;
#pragma unroll
    for (int pr = 0; pr < kRounds; ++pr) {
        const int pidx = wave + pr * DK_WAVES;   // = i * (TN / 2) + c / 2
        const int i = pidx / (TN / 2), c = (pidx % (TN / 2)) * 2;
        const int m = row0 + wrow + (i >> 1) * 16 + (i & 1);
        const int n = col0 + wcol + (c >> 1) * 16;
        if (pidx < kPairs && m < p.M && n < p.N) {
            Acc<OP> sum[2];
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int q = 0; q < Acc<OP>::kWords; ++q) {
                    int32_t v = 0;
#pragma unroll
                    for (int w8 = 0; w8 < DK_WAVES; ++w8)
                        v += red[w8 * kWaveWords + ((i * TN + c + e) * Acc<OP>::kWords + q) * 64 + lane];
                    sum[e].word(q) = v;
                }
            int32_t rc = 0;
            if (OP == OP_TERNARY) rc = p.cmul * p.rowc[m];
            const int32_t v0 = finalize<OP>(sum[0], p, rc);
            const int32_t v1 = finalize<OP>(sum[1], p, rc);
            const bool two = n + 1 < p.N;
            if (p.C != nullptr) {
                int32_t* dst = p.C + ((int64_t)m * p.ldc_m + (int64_t)n * p.ldc_n);
                if (pair_c && two) {
                    typedef int32_t i32x2 __attribute__((ext_vector_type(2)));
                    const i32x2 v = {v0, v1};
                    *reinterpret_cast<i32x2*>(dst) = v;
                } else {
                    dst[0] = v0;
                    if (two) dst[p.ldc_n] = v1;
                }
            }
            if (p.Cf != nullptr) {
                const float sc = p.scale[m];
                float f0 = __fmul_rn(sc, (float)v0), f1 = __fmul_rn(sc, (float)v1);
                if (p.bias != nullptr) {
                    const float bs = p.bias[m];
                    f0 = __fadd_rn(f0, bs);
                    f1 = __fadd_rn(f1, bs);
                }
                float* dst = p.Cf + ((int64_t)m * p.ldf_m + (int64_t)n * p.ldf_n);
                if (pair_f && two) {
                    typedef float f32x2 __attribute__((ext_vector_type(2)));
                    const f32x2 v = {f0, f1};
                    *reinterpret_cast<f32x2*>(dst) = v;
                } else {
                    dst[0] = f0;
                    if (two) dst[p.ldf_n] = f1;
                }
            }
        }
    }
}

// Few columns and a long K (fully connected layers at batch 5-128): chosen where even the 32 x 32 tiles of
// the problem number at most two per compute unit.  16-row tiles where 32-row tiles would leave compute
// units without a workgroup.  Measured for 4096 x N x 4608: N = 16 / 32 / 64 / 128 in 6.1 / 6.2 / 8.5 /
// 13.0 us against 17.1 / 17.5 / 17.7 / 20.4 us on the tiled kernel.  Returns 1 when the shape does not suit it.
template <int OP>
int launch_deepk(const GemmParams& p, hipStream_t stream) {
    // (the three-accumulator uniform two-bit basis is not a fully connected layer's operator; it keeps the tiled kernel)
    if constexpr (OP == OP_TWOBIT_UNIFORM) {
        return 1;
    } else {
    if (p.is_conv || p.N > 128 || p.Kw < 64) return 1;
    const int mode = tuning().gemm_deepk;   // 0 automatic, 1 always (where the shape fits), 2 never
    if (mode == 2) return 1;
    const int cus = compute_units();
    const int64_t tiles_n = ((int64_t)p.N + DK_BN - 1) / DK_BN;
    const int64_t t32 = (((int64_t)p.M + 31) / 32) * tiles_n;
    if (mode == 0 && t32 > 2 * (int64_t)cus) return 1;
    if (((int64_t)p.M + 15) / 16 * tiles_n > 0x7FFFFFF0LL) return 1;
    const LaunchTiming t = take_launch_timing();
    // (64-row tiles were measured too: never faster, 4096 x 128 x 4608 15.7 against 14.8 us)
    if (t32 >= cus) {
        const int tiles_m = (p.M + 31) / 32;
        hipExtLaunchKernelGGL((deepk_gemm_kernel<OP, 4>), dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * DK_WAVES), 0,
                              stream, t.start, t.stop, 0, p, tiles_m);
    } else {
        const int tiles_m = (p.M + 15) / 16;
        hipExtLaunchKernelGGL((deepk_gemm_kernel<OP, 2>), dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * DK_WAVES), 0,
                              stream, t.start, t.stop, 0, p, tiles_m);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
    }
}

template <int OP, int WM, int WN, int TM, int TN>
int launch_shape(const GemmParams& p, hipStream_t stream) {
    constexpr int BM = WM * 8 * TM;
    constexpr int BN = WN * 8 * TN;
    const int tiles_m = (p.M + BM - 1) / BM;
    const int64_t tiles_n = ((int64_t)p.N + BN - 1) / BN;
    const int64_t ntiles = (int64_t)tiles_m * tiles_n;
    if (ntiles > 0x7FFFFFF0LL) return -2;
    const unsigned grid = (unsigned)(((ntiles + 7) / 8) * 8);
    const LaunchTiming t = take_launch_timing();
    const StreamKArgs none{};
    if (p.is_conv)
        hipExtLaunchKernelGGL((plane_gemm_kernel<OP, WM, WN, TM, TN, true, false>), dim3(grid), dim3(64 * WM * WN), 0,
                              stream, t.start, t.stop, 0, p, tiles_m, (int)ntiles, none);
    else
        hipExtLaunchKernelGGL((plane_gemm_kernel<OP, WM, WN, TM, TN, false, false>), dim3(grid), dim3(64 * WM * WN),
                              0, stream, t.start, t.stop, 0, p, tiles_m, (int)ntiles, none);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Compute units of the current device (asked once per device index; concurrent first calls store the same value).
int compute_units() {
    static std::atomic<int> cache[16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    const bool cached = dev >= 0 && dev < 16;
    int v = cached ? cache[dev].load(std::memory_order_relaxed) : 0;
    if (v == 0) {
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
        if (cached) cache[dev].store(v, std::memory_order_relaxed);
    }
    return v;
}

// The even-share launch of the 64 x 64 tile (32 x 32 per wavefront, 4 x 4 accumulators per lane for the
// one-word operators).  Returns 1 when the problem or the workspace does not suit it (the caller then
// takes a tile-per-workgroup launch), 0 on success, negative on a launch error.
template <int OP, int TM, int TN>
int launch_even_share(const GemmParams& p, hipStream_t stream, const int always_per_cu = 0) {
    constexpr int WM = 2, WN = 2, NT = 256;
    constexpr int BM = WM * 8 * TM, BN = WN * 8 * TN;
    constexpr int64_t kTileBytes = (int64_t)TM * TN * Acc<OP>::kWords * NT * 4;
    if (p.ws == nullptr || p.ws_bytes <= (size_t)kEvenShareCounterBytes) return 1;
    const int tiles_m = (p.M + BM - 1) / BM;
    const int64_t tiles_n = ((int64_t)p.N + BN - 1) / BN;
    const int64_t ntiles = (int64_t)tiles_m * tiles_n;
    const int nst = (p.Kw + KT - 1) / KT;
    const int64_t units = ntiles * nst;
    if (ntiles > kEvenShareCounterBytes / 4 || units >= 0x7FFFFFFFLL) return 1;
    const int forced = always_per_cu > 0 ? always_per_cu : tuning().gemm_even_share;
    if (forced == 9 || forced == 10 || forced == 11) return 1;
    const int cus = compute_units();
    const int64_t fit = ((int64_t)p.ws_bytes - kEvenShareCounterBytes) / (2 * kTileBytes);
    int64_t G;
    if (forced >= 1 && forced <= 8) {
        G = (int64_t)cus * forced;
    } else {
        // Where the even shares of 64 x 64 tiles beat one 32 x 32 tile per workgroup (measured, us, plain -> even
        // shares): with few tiles and a long K, where the plain launch is one long chain of load latencies per
        // workgroup -- 256^2 x 32768 71 -> 32, 512^2 x 16384 37 -> 28, 256 x 2048 x 16384 (two tiles per
        // compute unit) 44 -> 39, 256 x 3072 x 32768 (three) 100 -> 91; not at K = 8192 (256 x 1024 x 8192
        // 20.4 -> 20.9, 256 x 3072 x 8192 27.9 -> 30.4) and not at K = 4096 (11.6 -> 16.1).
        const int64_t t32 = (((int64_t)p.M + 31) / 32) * (((int64_t)p.N + 31) / 32);
        if (ntiles >= 4 * (int64_t)cus || nst < 16) return 1;
        if (t32 < 8 * (int64_t)cus) {
            // (with at most two 32 x 32 tiles per compute unit launch_even_share_small is tried first and wins)
            const bool few_long = (nst >= 64 && t32 <= 2 * (int64_t)cus) || (nst >= 128 && t32 <= 3 * (int64_t)cus);
            if (!few_long) return 1;
        } else {
            // Beyond eight 32 x 32 tiles per compute unit the plain launch needs a second round of workgroups.
            // K >= 8192: 1536^2 77.1 -> 69.9, 1600^2 82.2 -> 76.2, 1472^2 73.2 -> 66.7.  K = 4096: only where
            // that round is thin (1536^2, one tile per unit left: 41.2 -> 40.2; 1664^2, 2.6 left: 45.0 -> 46.5;
            // 1792^2, 4.25 left: 50.0 -> 52.6); never where nothing is left (4096 x 512 x 4608: 38.0 -> 39.0).
            const int64_t left = t32 % (8 * (int64_t)cus);
            if (left == 0 || left > (nst >= 32 ? 4 : 1) * (int64_t)cus) return 1;
        }
        // About eight stages per workgroup, in whole multiples of the compute units (every unit then runs the
        // same number of equal shares), two to four per unit -- but never more than sixteen pieces per tile
        // nor fewer than four stages per piece.  Measured with 1 / 2 / 3 / 4 per unit: 256^2 x 32768 (16 tiles)
        // 31.8 / 39.2 / 55.0 / 61.5 us, 512^2 x 16384 36.6 / 28.5 / 31.5 / 34.5, 768^2 x 8192 41.0 / 29.7 /
        // 27.7 / 30.3, 333 x 777 x 5555 23.2 / 20.0 / 21.6 / 26.2, 1024^2 x 8192 61.0 / 40.9 / 39.3 / 36.6: the
        // partial sums of a tile cut into many short pieces all pass through the one workgroup that finishes it.
        int64_t per_cu = (units + 8 * (int64_t)cus - 1) / (8 * (int64_t)cus);
        per_cu = per_cu < 2 ? 2 : (per_cu > 4 ? 4 : per_cu);
        G = (int64_t)cus * per_cu;
        if (G > 16 * ntiles) G = 16 * ntiles;
        if (G > units / 4) G = units / 4;
    }
    if (G > units) G = units;
    G = (G + 7) & ~(int64_t)7;   // the XCD mapping wants a multiple of 8; workgroups without units return at once
    if (G > fit) G = fit & ~(int64_t)7;
    if (G < 8) return 1;
    StreamKArgs sk{};
    sk.counters = reinterpret_cast<int32_t*>(p.ws);
    sk.partial = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(p.ws) + kEvenShareCounterBytes);
    sk.nst = nst;
    sk.units = (int32_t)units;
    set_shares(sk, G);
    const LaunchTiming t = take_launch_timing();
    hipExtLaunchKernelGGL((plane_gemm_kernel<OP, WM, WN, TM, TN, false, true>), dim3((unsigned)G), dim3(NT), 0, stream,
                          t.start, t.stop, 0, p, tiles_m, (int)ntiles, sk);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Even shares of 32 x 32 tiles: for GEMMs with at most two of these tiles per compute unit and a long K, where
// a tile per workgroup is one long chain of load latencies on a mostly idle chip.  The shares are those of
// launch_even_share; the tile is the small one because its pieces hand over a quarter of the partial sums
// and its K loop runs the stages without tail tests.  Measured against the better of the plain launch and
// the 64 x 64 shares (us): 128 x 512 x 8192 20.3 -> 13.3, 256 x 1024 x 8192 20.3 -> 16.7, 256 x 2048 x 8192
// 23.6 -> 21.7 (256 x 3072 x 8192: 27.8 -> 28.3, not taken); 128 x 512 x 16384 24.9 -> 17.4, 256 x 1024 x 16384
// 28.2 -> 24.4, 256 x 2048 x 16384 38.9 -> 36.1; 128 x 512 x 32768 31.5 -> 25.2, 256 x 1024 x 32768 44.7 -> 38.4;
// nothing to gain at K = 4096.  About sixteen stages per workgroup, one to four workgroups per compute unit
// (128 x 512 x 16384 with 1 / 2 / 4 per unit: 17.4 / 20.7 / 32.7; 256 x 1024 x 16384: 36.7 / 26.3 / 24.4).
// Returns 0 = launched, 1 = not applicable, -1 = launch error.
template <int OP>
int launch_even_share_small(const GemmParams& p, hipStream_t stream) {
    constexpr int NT = 256, BM = 32, BN = 32;
    constexpr int64_t kTileBytes = (int64_t)2 * 2 * Acc<OP>::kWords * NT * 4;
    if (p.ws == nullptr || p.ws_bytes <= (size_t)kEvenShareCounterBytes) return 1;
    const int forced = tuning().gemm_even_share;
    if (forced != 0 && forced != 11) return 1;
    const int tiles_m = (p.M + BM - 1) / BM;
    const int64_t ntiles = (int64_t)tiles_m * (((int64_t)p.N + BN - 1) / BN);
    const int nst = (p.Kw + KT - 1) / KT;
    const int64_t units = ntiles * nst;
    if (ntiles > kEvenShareCounterBytes / 4 || units >= 0x7FFFFFFFLL) return 1;
    const int64_t cus = compute_units();
    if (forced == 0 && (nst < 32 || ntiles > 2 * cus)) return 1;
    int64_t per_cu = (units + 16 * cus - 1) / (16 * cus);
    per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
    int64_t G = cus * per_cu;
    if (G > units / 4) G = units / 4;   // at least four stages each
    G = (G + 7) & ~(int64_t)7;
    const int64_t fit = ((int64_t)p.ws_bytes - kEvenShareCounterBytes) / (2 * kTileBytes);
    if (G > fit) G = fit & ~(int64_t)7;
    if (G < 8) return 1;
    StreamKArgs sk{};
    sk.counters = reinterpret_cast<int32_t*>(p.ws);
    sk.partial = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(p.ws) + kEvenShareCounterBytes);
    sk.nst = nst;
    sk.units = (int32_t)units;
    set_shares(sk, G);
    const LaunchTiming t = take_launch_timing();
    hipExtLaunchKernelGGL((plane_gemm_kernel<OP, 2, 2, 2, 2, false, true>), dim3((unsigned)G), dim3(NT), 0, stream,
                          t.start, t.stop, 0, p, tiles_m, (int)ntiles, sk);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Whole tiles plus a split remainder (see StreamKArgs): for tile counts of q * CUs + r with a small q, where
// the plain launch leaves r compute units with q + 1 tiles and the others with q.  The q * CUs leading tiles
// go one to a workgroup; the r remaining tiles are cut into one even share per compute unit.
// Returns 0 = launched, 1 = not applicable, -1 = launch error.
template <int OP, int TM, int TN>
int launch_split_remainder(const GemmParams& p, hipStream_t stream) {
    constexpr int WM = 2, WN = 2, NT = 256;
    constexpr int BM = WM * 8 * TM, BN = WN * 8 * TN;
    constexpr int64_t kTileBytes = (int64_t)TM * TN * Acc<OP>::kWords * NT * 4;
    if (p.ws == nullptr || p.ws_bytes <= (size_t)kEvenShareCounterBytes) return 1;
    const int forced = tuning().gemm_even_share;
    if (forced != 0 && forced != 10) return 1;
    const int tiles_m = (p.M + BM - 1) / BM;
    const int64_t ntiles = (int64_t)tiles_m * (((int64_t)p.N + BN - 1) / BN);
    const int nst = (p.Kw + KT - 1) / KT;
    if (ntiles > kEvenShareCounterBytes / 4 || ntiles * nst >= 0x7FFFFFFFLL) return 1;
    const int cus = compute_units();
    const int64_t q = ntiles / cus, r = ntiles - q * cus;
    // Measured on 256 x N x K with N chosen for q = 1..7 and r = 16..192 (this launch's time over the plain
    // launch's): K = 9216: 0.88-0.95 for q = 2..6 and r <= 128, 0.96-0.99 at r = 192; K = 4608: 0.91-0.96 for
    // q = 4, 5, 7 and r <= 128, 0.95-0.985 for q = 3, 1.06 for q = 2 with r <= 32; K = 2304: 0.91 for q = 5,
    // 0.95 for q = 6 with r <= 64, 1.07-1.36 for q <= 4; K = 1152: 1.0-1.6.  The hand-over of the split tiles
    // has to hide behind at least q tiles of work.  At most eight workgroups of these tiles are resident per
    // compute unit, hence q <= 7.
    if (r == 0 || q < 1) return 1;
    if (forced == 0) {
        if (q > 7) return 1;
        if (nst >= 32) {
            if (q < 2 || r > cus / 2) return 1;
        } else if (nst >= 16) {
            if (q < 3 || r > cus / 2) return 1;
        } else if (nst >= 8) {
            if (q < 5 || q > 6 || r > cus / 4) return 1;
        } else {
            return 1;
        }
    }
    int64_t pieces = cus;
    if (pieces > r * nst / 2) pieces = (r * nst / 2) & ~(int64_t)7;
    const int64_t fit = ((int64_t)p.ws_bytes - kEvenShareCounterBytes) / (2 * kTileBytes);
    if (pieces > fit) pieces = fit & ~(int64_t)7;
    if (pieces < 8 || (q * cus) % 8 != 0) return 1;
    StreamKArgs sk{};
    sk.counters = reinterpret_cast<int32_t*>(p.ws);
    sk.partial = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(p.ws) + kEvenShareCounterBytes);
    sk.nst = nst;
    sk.units = (int32_t)(ntiles * nst);
    sk.whole = (int32_t)(q * cus);
    set_shares(sk, pieces);
    const LaunchTiming t = take_launch_timing();
    hipExtLaunchKernelGGL((plane_gemm_kernel<OP, WM, WN, TM, TN, false, true>), dim3((unsigned)(sk.whole + pieces)),
                          dim3(NT), 0, stream, t.start, t.stop, 0, p, tiles_m, (int)ntiles, sk);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Picks the workgroup shape, all 2 x 2 wavefronts.  Measured on this chip: the 64 x 64 tile (4 x 4
// accumulators per lane, six wavefronts per SIMD) matches the 128 x 128 tile (8 x 8 accumulators, three per
// SIMD) up to 8192^3 and beats it below about 16 K wavefront tiles of 64 x 64, where tile quantisation
// over 256 CUs matters; the large tile keeps a few per cent on very large problems with a shallow K
// (fewer operand re-reads).  Below that size, and given a workspace, the 64 x 64 tile runs under the
// even-share schedule, which has no tile quantisation at all, or the 32 x 32 tile runs with only the
// remainder of its tile count split (launch_even_share and launch_split_remainder say where each pays).
// Otherwise: below about a thousand 64 x 64 wavefront tiles the 32 x 32 tile (2 x 2 accumulators) puts four
// times as many wavefronts to work (4096 x 64 x 4608: 25 -> 18 us, 1536^2 x 4096: 53 -> 41 us) but reads LDS
// once per 8 instruction pairs.
template <int OP, int TM, int TN>
int launch_op(const GemmParams& p, hipStream_t stream) {
    constexpr int WTM = 8 * TM, WTN = 8 * TN;
    const int64_t wave_tiles = (((int64_t)p.M + WTM - 1) / WTM) * (((int64_t)p.N + WTN - 1) / WTN);
    // (Even shares for the large tile, three workgroups per compute unit, were measured as well: the kernel
    // then needs 179 registers, eight of them spilled to stay at three wavefronts per SIMD, and 8192^3 took
    // 1826 instead of 1605 us.)
    if (wave_tiles >= 16 * 1024 && p.M > WTM) return launch_shape<OP, 2, 2, TM, TN>(p, stream);
    if (!p.is_conv) {
        int rc = launch_deepk<OP>(p, stream);
        if (rc <= 0) return rc;
        // Three to eight 32 x 32 tiles per compute unit: splitting only the remainder beats the even shares
        // of 64 x 64 tiles where both apply (1280^2 x 8192: 47.5 against 54.8 us); with fewer tiles and a very
        // long K the even shares come first.
        const int64_t t32 = (((int64_t)p.M + 31) / 32) * (((int64_t)p.N + 31) / 32);
        const int64_t cus = compute_units();
        const bool split_first = t32 >= 3 * cus && t32 < 8 * cus;
        if (wave_tiles < 1024) {
            rc = launch_even_share_small<OP>(p, stream);
            if (rc <= 0) return rc;
        }
        if (split_first) {
            rc = launch_split_remainder<OP, 2, 2>(p, stream);
            if (rc <= 0) return rc;
        }
        rc = launch_even_share<OP, TM / 2, TN / 2>(p, stream);
        if (rc <= 0) return rc;
        if (!split_first && wave_tiles < 1024) {
            rc = launch_split_remainder<OP, 2, 2>(p, stream);
            if (rc <= 0) return rc;
        }
    }
    // One tile per workgroup: the middle tile (64 x 64 for the one-word operators) or the 32 x 32 tile.  Fully
    // balanced, the middle tile is about 10 % faster (2048^3 33.1 against 36.6 us, 3072^3 94.3 against 104.6),
    // but a compute unit runs whole tiles, ceil(tiles / CUs) of them on the busiest unit, and that rounding
    // costs the larger tile more: 2560^3 (6.25 middle tiles per unit) 70.9 against 63.9 us, 512 x 12544 x 2304
    // (6.125) 62.7 against 57.8, 1792^2 x 4096 (3.06) 58.1 against 50.6; 1536 x 2048 x 2048 (3 exactly) 27.1
    // against 29.0.  Below three middle tiles per unit the small tile keeps more wavefronts at work
    // (2048 x 1024 x 8192, two per unit: 69.5 against 61.0 us).
    const int64_t units_cu = compute_units();
    const int64_t t_small = (((int64_t)p.M + 31) / 32) * (((int64_t)p.N + 31) / 32);
    auto busiest_over_mean = [&](int64_t tiles) {
        return (double)(((tiles + units_cu - 1) / units_cu) * units_cu) / (double)tiles;
    };
    // (The convolution front end keeps its per-tile addressing cheaper on the middle tile: from 1024 of them on
    // it wins whatever the rounding -- 128 x 50176 x 1152, 6.125 per unit: 37.4 against 40.9 us.)
    const bool middle = p.is_conv ? wave_tiles >= 1024
                                  : wave_tiles >= 3 * units_cu &&
                                        busiest_over_mean(wave_tiles) <= 1.10 * busiest_over_mean(t_small);
    if (middle) return launch_shape<OP, 2, 2, TM / 2, TN / 2>(p, stream);
    return launch_shape<OP, 2, 2, 2, 2>(p, stream);
}

}  // namespace

int launch_ternary_gemm_even_share(const GemmParams& p, int wgs_per_cu, hipStream_t stream) {
    if (p.M == 0 || p.N == 0) return 0;
    return launch_even_share<OP_TERNARY, 4, 4>(p, stream, wgs_per_cu);
}

int launch_gemm(const GemmParams& p, int op, hipStream_t stream) {
    if (p.M == 0 || p.N == 0) return 0;
    // (the measurement switch that forces the K-splitting kernel also forces it over the matrix-vector kernel)
    if (skinny_supported(p, op) && tuning().gemm_deepk != 1) return launch_skinny_gemm(p, stream);
    switch (op) {
        case OP_TERNARY: return launch_op<OP_TERNARY, 8, 8>(p, stream);
        case OP_TWOBIT_TERNARY: return launch_op<OP_TWOBIT_TERNARY, 8, 8>(p, stream);
        case OP_TWOBIT_UNIFORM: return launch_op<OP_TWOBIT_UNIFORM, 8, 4>(p, stream);
        case OP_XOR_PAIR: return launch_op<OP_XOR_PAIR, 8, 8>(p, stream);
        default: return -3;
    }
}

}  // namespace fatnn
