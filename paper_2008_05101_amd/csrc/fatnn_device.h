// Shared declarations of the HIP translation units (kernels + host layer).
// gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

namespace fatnn {

constexpr int kWave = 64;

// Places the next instruction at an address that is 4 modulo 8.  The hot loops are long runs
// of 8-byte VOP3 instructions (v_bitop3_b32, v_bcnt_u32_b32); measured on gfx950, such a run
// issues about 10 % faster when its instructions straddle the 8-byte boundaries than when
// they sit on them (same instructions, same registers, only the code address differs), so
// each run is started at the faster phase.  Costs one or two s_nop.
#define FATNN_VOP3_RUN_PHASE() asm volatile(".p2align 3\n\ts_nop 0")

// A packed element pair: two 32-bit plane words covering 32 consecutive k.
using plane2 = uint2;

enum PackKind : int {
    PACK_ACT = 0,      // .x = (l == 2), .y = (l >= 1)
    PACK_WEIGHT = 1,   // .x = (l == 2), .y = (l != 1)
    PACK_TWOBIT = 2,   // .x = bit 1,    .y = bit 0 of a code in {0,1,2,3}
    PACK_BINARY = 3    // one bit per element, 64 elements per word pair (.x = first 32)
};

// Source addressing of a level tensor: element (row, k) lives at
//   levels[row_off(row) + k_off(k)]; only the gathering kernel uses the general form.
struct GatherDesc {
    // row = (r0 * n1 + r1):   row offset = r0 * rs0 + r1 * rs1
    int64_t n1, rs0, rs1;
    // k = (k0 * C + c):       k offset  = k0 * ks0 + c * ks1
    int64_t C, ks0, ks1;
};

int launch_pack_contiguous(const int8_t* levels, int64_t rows, int64_t K, int kind, plane2* packed,
                           int32_t* n_invalid, hipStream_t stream);
int launch_pack_gather(const int8_t* levels, int64_t rows, int64_t K, GatherDesc g, int kind,
                       plane2* packed, int32_t* n_invalid, hipStream_t stream);
// Quantize-and-pack from float32: level = (p >= t1) + (p >= t2); nan_lo = low plane bit given to NaN.
int launch_quantize_pack(const float* x, int64_t rows, int64_t K, int kind, float t1, float t2, uint32_t nan_lo,
                         plane2* packed, int32_t* n_invalid, hipStream_t stream);
int launch_quantize_pack_bordered(const float* x, int64_t B, int64_t H, int64_t W, int64_t C, int border,
                                  plane2 border_word, int64_t slack_pixels, float t1, float t2, uint32_t nan_lo,
                                  plane2* packed, int32_t* n_invalid, hipStream_t stream);
int launch_fill_words(plane2* dst, int64_t count, plane2 word, hipStream_t stream);
int launch_interleave_weights(const plane2* packed, int64_t rows, int64_t Kw, plane2* inter, hipStream_t stream);
int launch_pack_binary(const int8_t* bits, int64_t rows, int64_t K, plane2* packed, int32_t* n_invalid,
                       hipStream_t stream);
int launch_row_constants(const plane2* packed, int64_t rows, int64_t Kw, int32_t* nnz, int32_t* npos,
                         hipStream_t stream);

enum GemmOp : int {
    OP_TERNARY = 0,        // Eq. 3 in its reduced form: 2 logic + 2 popcount per word pair
    OP_TWOBIT_TERNARY = 1, // Eq. 2, alpha = beta = (1/2,1/2): 4 xor + 4 popcount, one accumulator
    OP_TWOBIT_UNIFORM = 2, // Eq. 2, alpha = beta = (1,2):     4 xor + 4 popcount, three accumulators
    OP_XOR_PAIR = 3        // Eq. 1 / Eq. 4 alone: popcount(x ^ y) word by word, C = K - cmul * sum
};

struct GemmParams {
    const plane2* W;        // [M][Kw]
    const plane2* A;        // GEMM: [N][Kw];  conv: [B][H][Wd][Cw]
    const int32_t* rowc;    // per-row constant source (nnz or npos), ternary op only
    int32_t cmul;           // C = cmul * rowc[m] - P'        (ternary)
    int32_t K;              // true element count (two-bit epilogues)
    int32_t M, N, Kw;
    int32_t* C;             // may be null
    int64_t ldc_m, ldc_n;   // element strides of C along m and n
    float* Cf;              // may be null
    int64_t ldf_m, ldf_n;
    const float* scale;
    const float* bias;
    // convolution front end (is_conv != 0)
    int32_t is_conv;
    int32_t B, H, Wd, Cw, Ho, Wo, R, S, stride, pad;
    int32_t cw_shift;       // log2(Cw) when Cw is a power of two, else -1
    uint32_t pad_x, pad_y;  // plane words of a padded tap (value 0)
    // even-share schedule (GEMM only): device workspace whose first kEvenShareCounterBytes are zero, or null
    void* ws;
    size_t ws_bytes;
};

// Workspace of the even-share GEMM schedule: tile counters (one int32 per 64 x 64 tile, at most 16384 tiles)
// followed by the hand-over slots.
constexpr int64_t kEvenShareCounterBytes = 64 * 1024;

int launch_gemm(const GemmParams& p, int op, hipStream_t stream);
// The ternary GEMM under the even-share schedule whatever its size, wgs_per_cu workgroups per compute unit
// (fewer if the workspace in p is smaller).  Returns 1 if the workspace cannot serve the problem.
int launch_ternary_gemm_even_share(const GemmParams& p, int wgs_per_cu, hipStream_t stream);
bool skinny_supported(const GemmParams& p, int op);          // ternary GEMM with a handful of columns (matrix-vector shaped)
int launch_skinny_gemm(const GemmParams& p, hipStream_t stream);

// Measurement hook (fatnn_time_next_launch): events that the next GEMM / convolution
// kernel launch of this thread attaches to the dispatch itself; consumed by that launch.
struct LaunchTiming {
    hipEvent_t start, stop;
};
LaunchTiming take_launch_timing();

// Measurement switches (process-wide; see fatnn_set_tuning).  Initial values come from the environment,
// read once: FATNN_CONV_KERNEL=tiled, FATNN_STREAM_WPS=n, FATNN_STREAM_U7=0|1|2.
struct Tuning {
    bool force_tiled;   // convolutions go to the LDS-tiled kernel even where the streaming one applies
    int stream_wps;     // wavefronts per SIMD of the streaming kernel (0 = planned)
    int u7_mode;        // seven-pixel groups: 0 off, 1 by the size rule, 2 wherever a kernel exists
    int gemm_even_share;  // even-share GEMM schedule: 0 automatic, 1..8 workgroups per CU forced, 9 never,
                          // 10 whole tiles + split remainder wherever there is a remainder, 11 even shares of
                          // 32 x 32 tiles whatever the size
    int gemm_deepk;       // few-column / long-K kernel: 0 automatic, 1 wherever the shape fits, 2 never
};
Tuning tuning();
// a negative value keeps the current one
void set_tuning(int force_tiled, int stream_wps, int u7_mode, int gemm_even_share, int gemm_deepk);

// Column-streaming convolution (weights resident in registers, activations through
// the scalar cache).  Input: bordered packed activations [B][Hp][Wp][Cw] (+ slack),
// i.e. padding is physical.  Output is NHWC: element (n, m) at n * ldc_n + m.
struct StreamParams {
    const plane2* Wi;       // interleaved weights: [ceil(M/64)][Kw][64] (lane-contiguous)
    const uint32_t* A;      // bordered packed activations as dwords (hi, lo pairs)
    const int32_t* rowc;
    int32_t cmul;
    int32_t K;
    int32_t M, Kw;
    int32_t* C;
    float* Cf;
    int32_t ldc;            // elements between consecutive output pixels (= output channels)
    uint32_t out_bytes;     // size of each output tensor in bytes (below 4 GiB)
    const float* scale;
    const float* bias;
    int32_t Hp, Wp, Ho;     // bordered input height / width, output height
    int32_t wgroups, tailU; // groups of U output pixels per output row; pixels in the last one
    int32_t gq, gr;         // groups per range of the grid: range r owns gq + (r < gr)
    int32_t xoff;           // physical border minus the convolution's padding (0 or 1)
    // Layer-chaining epilogue (Xn != nullptr): affine, optional skip and ReLU in fp32, then the
    // next layer's activation quantizer and packing straight into its bordered input buffer.
    plane2* Xn;             // [B][nHp][nWp][nCw] word pairs, ring already initialised
    int32_t nHp, nWp, nCw, nborder;
    const float* skip;      // fp32 NHWC [B][Ho][Wo][M] or null
    float t1, t2;           // level = (f >= t1) + (f >= t2)
    uint32_t nan_lo;
    int32_t relu;
};

bool stream_supported(int op, int R, int S, int Cw, int stride);
// out_rows = batch x output height, Wo = output width; wgroups, tailU, gq and gr are filled in here.
int launch_stream_conv(const StreamParams& p, int op, int R, int Cw, int stride, int64_t out_rows, int64_t Wo,
                       hipStream_t stream);

// Roofline probes (peaks.hip): register-resident issue-rate loop of the method's instruction pair and
// HBM streaming passes.  kind of the VALU probe: 0 pair with vector operands, 1 pair with the data word in
// an SGPR, 2 popcount alone, 3 three-input logic alone, 4 plain xor.  kind of the HBM probe: 0 read, 1 write,
// 2 copy.  Both consume the launch-timing hook.
int probe_pairs_per_iteration();
int launch_valu_probe(int kind, int blocks, int iters, const uint32_t* seed, int32_t* sink, hipStream_t stream);
int launch_hbm_probe(int kind, void* dst, const void* src, size_t bytes, int blocks, uint32_t* sink,
                     hipStream_t stream);

// Bordered activation packing: levels NHWC [B][H][W][C] -> [B][H+2*border][W+2*border][C/32]
// word pairs, ring pixels = border_word; `slack_pixels` more pixels of border_word follow.
int launch_pack_bordered(const int8_t* levels, int64_t B, int64_t H, int64_t W, int64_t C, int border, int kind,
                         plane2 border_word, int64_t slack_pixels, plane2* packed, int32_t* n_invalid,
                         hipStream_t stream);

}  // namespace fatnn
