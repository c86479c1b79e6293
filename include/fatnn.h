/*
 * fatnn.h -- C ABI of the MI355X (gfx950) ternary GEMM / convolution library.
 *
 * The library evaluates the reduced-complexity ternary inner product of FATNN
 * (arXiv 2008.05101, Section 3.3): two ternary vectors are stored in the 2-bit
 * codec of Table 1 (popcount(codec) = value + 1), multiplied with a handful of
 * bitwise operations (Eq. 4-7) and accumulated with one popcount per packed word
 * (Eq. 3, Algorithm 1), instead of the four binary inner products that the
 * conventional decomposition (Eq. 2 with two bits per operand) needs.
 *
 * Conventions common to every entry point
 *   - Tensors are addressed through plain pointers.  Every tensor pointer is a
 *     DEVICE pointer owned by the caller; the library never allocates, frees or
 *     keeps it.  `dims` arrays and scalars are host values.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued asynchronously on it; nothing synchronises.
 *   - The return value is a fatnn_status.  Argument errors are found on the
 *     host before any GPU call, so they are reported even with no GPU present.
 *     No entry point throws or aborts.
 *   - Inputs are LEVEL INDICES l in {0,1,2} (int8), l = popcount of the paper's
 *     codec.  Weights mean l-1 in {-1,0,+1}.  Activations mean l-1 (FATNN_SYM) or
 *     l in {0,1,2} (FATNN_RELU, the paper's second constraint in Section 3.3).
 *   - Inputs outside that set break the paper's first constraint (Section 3.3).  The
 *     packing calls run asynchronously and cannot return that fact; they ADD the
 *     number of such elements to the device counter `n_invalid` and pack them as
 *     the value 0.  FATNN_ERR_LEVEL is the status for "the counter came back
 *     non-zero": fatnn_level_status(count) forms it, and the Python binding raises
 *     it when called with check_levels=True (which reads the counter back, i.e.
 *     synchronises).
 *   - Apart from the two measurement hooks at the end (fatnn_set_tuning, process-wide
 *     atomics; fatnn_time_next_launch, per thread) the library keeps no state, and
 *     every call is re-entrant.
 *   - Zero-sized problems (no rows / no columns / no batch) succeed and launch
 *     nothing.  K (or Cin) must be at least 1.
 *
 * Packed layout ("plane words"): a row of K elements becomes Kw = ceil(K/32)
 * pairs of 32-bit words; bit e of a pair's words belongs to element 32*kw + e.
 *     activations: .x = (l == 2),  .y = (l >= 1)      the two codec bits of Table 1
 *                                                     with 0 spelled 01
 *     weights:     .x = (l == 2),  .y = (l != 1)      sign bit and non-zero bit; the
 *                                                     latter is the complement of
 *                                                     Eq. 6's mask, fixed after
 *                                                     training like the paper's
 *   Tail elements (k >= K) are packed as the value 0.  A packed weight buffer
 *   ends with two int32 per row (count of non-zero weights, count of +1
 *   weights), from which the kernels form Eq. 3's "- N" term and the ReLU-mode
 *   constant ("add a copy of the weights", Section 3.3).
 */
#ifndef FATNN_H
#define FATNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FATNN_OK = 0,
    FATNN_ERR_NULL = -1,        /* a required pointer is NULL                         */
    FATNN_ERR_SHAPE = -2,       /* negative / zero / inconsistent dimension           */
    FATNN_ERR_LEVEL = -3,       /* an input outside the paper's level set: see below  */
    FATNN_ERR_ALIGN = -4,       /* pointer not aligned as documented                  */
    FATNN_ERR_SIZE = -5,        /* buffer too small, or dimension beyond the limits   */
    FATNN_ERR_UNSUPPORTED = -6, /* valid but not implemented (never a wrong answer)   */
    FATNN_ERR_HIP = -7          /* the HIP runtime refused a launch                   */
} fatnn_status;

enum { FATNN_WEIGHT = 0, FATNN_ACT = 1 };                 /* role     */
enum { FATNN_SYM = 0, FATNN_RELU = 1 };                   /* act_mode */
enum {                                                    /* layout of a level tensor, dims[4]        */
    FATNN_ROWMAJOR_K = 0, /* dims = {rows, K, 1, 1}: [rows][K], K contiguous                          */
    FATNN_NHWC = 1,       /* dims = {B, H, W, C}: rows = B*H*W pixels, K = C   (activations)          */
    FATNN_OHWI = 2,       /* dims = {O, R, S, C}: rows = O, K = R*S*C, c innermost (conv weights)     */
    FATNN_OIHW = 3,       /* dims = {O, C, R, S}: same packed result as OHWI (gathering, slow path)   */
    FATNN_NCHW = 4        /* dims = {B, C, H, W}: same packed result as NHWC (gathering, slow path)   */
};
enum { FATNN_X_PLAIN = 0, FATNN_X_BORDERED = 1, FATNN_X_BORDERED1 = 2 };  /* packed conv activations */
enum { FATNN_BASIS_TERNARY = 0, FATNN_BASIS_UNIFORM = 1, FATNN_BASIS_XNOR_ONLY = 2 };  /* see fatnn_twobit_gemm */

/* Largest supported extents: rows, columns < 2^31; K <= 2^24 (keeps |C| <= 2K exact in fp32 too). */
#define FATNN_MAX_K (1 << 24)

/* ceil(K / 32): plane-word pairs per packed row.  Returns -1 for K < 1. */
int64_t fatnn_words_per_row(int64_t K);

/* Bytes of a packed buffer of `rows` rows of K elements.  role = FATNN_WEIGHT adds
 * the per-row constants (see file header).  Returns 0 on invalid arguments.
 * Layout: rows*Kw pairs of uint32, then (weights only) at the next multiple of
 * 256 bytes int32 nnz[rows] followed by int32 npos[rows], then at the next multiple
 * of 256 bytes the lane-interleaved copy (fatnn_weight_interleaved_offset). */
size_t fatnn_packed_bytes(int role, int64_t rows, int64_t K);

/* Byte offset of the per-row constants inside a packed weight buffer. */
size_t fatnn_weight_consts_offset(int64_t rows, int64_t K);

/* Byte offset of the second, lane-interleaved copy of the plane words inside a packed
 * weight buffer: [ceil(rows/64)][Kw][64] pairs, rows past the end zero.  The
 * column-streaming convolution kernel reads the weights of 64 output channels with
 * one coalesced load per k-word from it. */
size_t fatnn_weight_interleaved_offset(int64_t rows, int64_t K);

/*
 * Algorithm 1, step 1 (data packing), from level indices.
 *   levels        device, int8, laid out as `layout` / `dims` say.
 *   role          FATNN_WEIGHT or FATNN_ACT (selects the plane meaning above; for
 *                 weights the per-row constants are computed too -- the
 *                 precomputation the paper does once after training, Section 3.3).
 *   packed        device, 16-byte aligned, at least fatnn_packed_bytes() bytes.
 *   n_invalid     device int32 or NULL.  The number of elements outside {0,1,2}
 *                 is ADDED to it (the caller zeroes it); such elements are packed
 *                 as the value 0.  The paper's first constraint makes them an
 *                 input error; a caller that cares reads the counter back.
 * NHWC / OHWI / OIHW / NCHW need C to be a multiple of 32 so that every pixel /
 * filter tap starts on a word boundary.
 */
int fatnn_pack_ternary(const int8_t *levels, int layout, const int64_t dims[4], int role,
                       void *packed, size_t packed_bytes, int32_t *n_invalid, void *stream);

/*
 * The same packing for convolution inputs, into the BORDERED layout
 *     [B][H + 2*border][W + 2*border][C/32] word pairs  (+ FATNN_BORDER_SLACK_PIXELS pixels),
 * where the ring of `border` pixels around every image and the slack behind the last
 * image hold the VALUE 0 under `act_mode` (level 1 in FATNN_SYM, level 0 in FATNN_RELU).
 * With border = the convolution's padding no tap ever falls outside the stored image,
 * which lets fatnn_ternary_conv2d run its fastest kernel; border = 0 is the plain
 * pixel order plus the slack (for 1x1 convolutions).
 *   levels   device int8, NHWC, dims = {B, H, W, C}, C a multiple of 32, 16-byte aligned
 *   packed   device, 16-byte aligned, at least fatnn_bordered_act_bytes() bytes
 */
#define FATNN_BORDER_SLACK_PIXELS 64
size_t fatnn_bordered_act_bytes(int64_t B, int64_t H, int64_t W, int64_t C, int border);
int fatnn_pack_ternary_bordered(const int8_t *levels, const int64_t dims[4], int border, int act_mode,
                                void *packed, size_t packed_bytes, int32_t *n_invalid, void *stream);

/*
 * Algorithm 1, step 1 as written: quantize full-precision data with the learned step
 * sizes and pack.  Weights and real-valued (FATNN_SYM) activations use the weight
 * quantizer of Eq. 8 / Eq. 9, level = Q^w(p) + 1; non-negative (FATNN_RELU) activations
 * use Eq. 10 (its misprinted parenthesis read as clip((p - alpha1) / alpha2, 0, 1)),
 * level = Q^a(p).  Rounding is round-half-to-even and every operation of the formulas
 * is a float32 operation; the kernel compares against the exact float32 break points
 * of those formulas, so the result equals normalise-saturate-round bit for bit.
 *   x             device float32; layout FATNN_ROWMAJOR_K, FATNN_NHWC or FATNN_OHWI
 *                 (K contiguous), 4-byte aligned (16-byte for the bordered form)
 *   alpha1/2      step sizes, finite and > 0 (else FATNN_ERR_SHAPE); act_mode is ignored
 *                 for role FATNN_WEIGHT
 *   n_invalid     NaN inputs are counted there and packed as the value 0
 * Buffers and sizes as for fatnn_pack_ternary / fatnn_pack_ternary_bordered.
 */
int fatnn_quantize_pack(const float *x, int layout, const int64_t dims[4], int role, int act_mode,
                        float alpha1, float alpha2, void *packed, size_t packed_bytes, int32_t *n_invalid,
                        void *stream);
int fatnn_quantize_pack_bordered(const float *x, const int64_t dims[4], int border, int act_mode,
                                 float alpha1, float alpha2, void *packed, size_t packed_bytes,
                                 int32_t *n_invalid, void *stream);

/*
 * Ternary GEMM through Eq. 3:  C[m][n] = sum_k w[m][k] * a[n][k].
 *   Wp            packed weights  [M][Kw] (+ constants), from fatnn_pack_ternary(role WEIGHT)
 *   Ap            packed activations [N][Kw], from fatnn_pack_ternary(role ACT)
 *   C             int32 [M][ldc], ldc >= N, or NULL
 *   Cf            fp32  [M][ldcf], ldcf >= N, or NULL:  Cf = scale[m] * float(C) (+ bias[m]);
 *                 the single high-precision coefficient of the paper's first
 *                 constraint, per output channel.  scale is required when Cf is
 *                 given; bias may be NULL.  At least one of C, Cf must be given.
 */
int fatnn_ternary_gemm(const void *Wp, const void *Ap, int64_t M, int64_t N, int64_t K, int act_mode,
                       int32_t *C, int64_t ldc, const float *scale, const float *bias, float *Cf,
                       int64_t ldcf, void *stream);

/*
 * Ternary convolution as an implicit GEMM (Supplementary S1: im2col + gemm, here
 * without materialising the matrix).
 *   Wp            packed weights from layout OHWI/OIHW: [Cout][R*S*Cin/32] (+ constants)
 *   Xp, x_layout  packed activations: FATNN_X_PLAIN = [B][H][W][Cin/32] from
 *                 fatnn_pack_ternary (NHWC/NCHW); FATNN_X_BORDERED = the bordered layout of
 *                 fatnn_pack_ternary_bordered with border == pad and the same act_mode;
 *                 FATNN_X_BORDERED1 = that layout with border 1 whatever pad is (a 1x1,
 *                 pad 0 convolution reading the buffer a 3x3, pad 1 convolution also reads)
 *   Y, Yf         int32 / fp32 NHWC outputs [B][Ho][Wo][Cout], Ho = (H + 2*pad - R)/stride + 1
 *   Padding is the VALUE 0 in either act_mode.
 * Supported: R = S in {1, 3}, stride in {1, 2}, pad in {0, 1} with pad <= R/2,
 * Cin a multiple of 32; anything else returns FATNN_ERR_UNSUPPORTED.
 */
int fatnn_ternary_conv2d(const void *Wp, const void *Xp, int x_layout, int64_t B, int64_t Cin, int64_t H,
                         int64_t W, int64_t Cout, int R, int S, int stride, int pad, int act_mode, int32_t *Y,
                         const float *scale, const float *bias, float *Yf, void *stream);

/*
 * Layer chaining (Supplementary S1: batch norm folded into the layer, ReLU and the skip
 * connection fused with the packing of the next layer's input).  Same convolution as
 * fatnn_ternary_conv2d on a bordered input (x_layout FATNN_X_BORDERED or _BORDERED1), but instead of the int32 result it produces
 *     f = scale[m] * C (+ bias[m]) (+ skip[n][m]),  f = max(f, 0) if relu != 0      (fp32, one
 *                                                   rounding per operation)
 *     level = quantizer of the NEXT layer applied to f: Eq. 9 for out_act_mode FATNN_SYM,
 *             Eq. 10 for FATNN_RELU, with step sizes alpha1, alpha2 (as fatnn_quantize_pack)
 * and writes the levels, packed, into the interior of the next layer's bordered input
 *     Xnext = [B][Ho + 2*out_border][Wo + 2*out_border][Cout/32] (+ slack),
 * whose ring must have been initialised once with fatnn_bordered_act_init (the ring is
 * never written here).  Yf (optional, NHWC fp32) receives f, e.g. as the next block's skip
 * input.  skip (optional) is NHWC fp32 [B][Ho][Wo][Cout].  Cout must be a multiple of 32.
 * Shapes the streaming kernel does not cover (filter 1 or 3, stride 1 or 2, Cin in {64, 128,
 * 256, 512}), and calls whose input, fp32 output or next-layer buffer reaches 4 GiB, return
 * FATNN_ERR_UNSUPPORTED.  A NaN in f: ReLU turns it into 0 (the maximum of NaN and 0); without
 * ReLU it is stored as NaN and gets the level the quantizer formula gives a NaN.
 */
int fatnn_bordered_act_init(void *packed, size_t packed_bytes, int64_t B, int64_t H, int64_t W, int64_t C,
                            int border, int act_mode, void *stream);
int fatnn_ternary_conv2d_chain(const void *Wp, const void *Xp, int x_layout, int64_t B, int64_t Cin, int64_t H,
                               int64_t W, int64_t Cout, int R, int S, int stride, int pad, int act_mode,
                               const float *scale, const float *bias, const float *skip, int relu,
                               float alpha1, float alpha2, int out_act_mode, int out_border, void *Xnext,
                               size_t xnext_bytes, float *Yf, void *stream);

/*
 * Conventional two-bit path (Eq. 2 with two bit-planes per operand and the binary
 * inner product of Eq. 1): four logic operations and four popcounts per packed
 * word pair where Eq. 3 needs two and two.  It exists so the paper's O(4N) ->
 * O(2N) claim (Remark 1) can be measured on the same chip with the same tiling.
 *
 * Codes q = 2*b1 + b0 in {0,1,2,3}; plane words .x = b1, .y = b0; tail bits 0.
 * fatnn_pack_twobit takes the same layouts, roles and buffer sizes as
 * fatnn_pack_ternary (role WEIGHT adds the interleaved copy; the constants are unused).
 * The value of a code is  alpha0*(2*b0-1) + alpha1*(2*b1-1):
 *   FATNN_BASIS_TERNARY  alpha = (1/2, 1/2): 00,01,10,11 -> -1,0,0,+1 (Table 1's codec)
 *   FATNN_BASIS_UNIFORM  alpha = (1, 2):     00,01,10,11 -> -3,-1,+1,+3
 * C[m][n] = sum_k value(w) * value(a), int32.
 *   FATNN_BASIS_XNOR_ONLY  is not a basis but the ablation of the paper's Table 4: on Table 1's
 *       codecs it evaluates Eq. 3 with the xnor rule of Eq. 4 ALONE, C = popcount(xnor) - K, i.e.
 *       without the "extra bit operations" of Eq. 5-7.  It is wrong whenever a weight is 0 (it
 *       treats 0 * a as the value of a's codec xnor 01) and exists only to time those operations.
 */
int fatnn_pack_twobit(const int8_t *codes, int layout, const int64_t dims[4], int role, void *packed,
                      size_t packed_bytes, int32_t *n_invalid, void *stream);
int fatnn_twobit_gemm(const void *Wp, const void *Ap, int64_t M, int64_t N, int64_t K, int basis,
                      int32_t *C, int64_t ldc, void *stream);
/* Bordered packing of two-bit codes; the ring holds code 01 (value 0 in the TERNARY basis). */
int fatnn_pack_twobit_bordered(const int8_t *codes, const int64_t dims[4], int border, void *packed,
                               size_t packed_bytes, int32_t *n_invalid, void *stream);
/* TERNARY basis only (the padded taps need a code of value 0). */
int fatnn_twobit_conv2d(const void *Wp, const void *Xp, int x_layout, int64_t B, int64_t Cin, int64_t H,
                        int64_t W, int64_t Cout, int R, int S, int stride, int pad, int basis, int32_t *Y,
                        void *stream);

/*
 * Binary networks (Eq. 1): x . y = 2 * popcount(xnor(x, y)) - N for x, y in {-1,+1}^N, one bit per
 * element (0 stands for -1).  The paper times binary layers next to ternary and 2-bit ones
 * (Table 3, Tables S1-S2); this is that comparison kernel, on the same tiling.
 *   bits    device int8 [rows][K] with values 0 / 1 (others are counted in *n_invalid and packed as 0)
 *   packed  [rows][ceil(K/64)] word pairs, 64 elements per pair, fatnn_binary_packed_bytes() bytes
 *   C       int32 [M][ldc]
 */
size_t fatnn_binary_packed_bytes(int64_t rows, int64_t K);
int fatnn_pack_binary(const int8_t *bits, int64_t rows, int64_t K, void *packed, size_t packed_bytes,
                      int32_t *n_invalid, void *stream);
int fatnn_binary_gemm(const void *Wb, const void *Ab, int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc,
                      void *stream);

/*
 * The three GEMM calls above with a workspace, for problems whose tiles do not fill the 256 compute units
 * evenly (a few hundred tiles, or few tiles with a long K: fully connected layers at batch 17-128, which
 * Supplementary S1 treats as convolutions whose filter covers the whole feature map).  Same arguments,
 * results identical bit for bit; with the workspace the library may cut the K loops of all tiles, or of the
 * tiles left over after whole rounds on the compute units, into equal shares for the workgroups and combine
 * the partial popcount sums of Eq. 3 through it.
 *   workspace        device, 16-byte aligned, or NULL (then exactly the plain call)
 *   workspace_bytes  any size; fatnn_gemm_workspace_bytes() lets every shape use the full schedule, a
 *                    smaller one limits the number of workgroups, one below 128 KiB is not used at all
 * The first 64 KiB of the workspace (tile counters) must be zero before the first call;
 * fatnn_gemm_workspace_init zeroes the whole workspace with a fill kernel, which is safe to capture into a
 * HIP graph.  Every call leaves the counters zero again, so one initialisation serves any number of calls.
 * Calls that share a workspace must be ordered (same stream, or events): they would race on it otherwise.
 */
size_t fatnn_gemm_workspace_bytes(void);
int fatnn_gemm_workspace_init(void *workspace, size_t workspace_bytes, void *stream);
int fatnn_ternary_gemm_ws(const void *Wp, const void *Ap, int64_t M, int64_t N, int64_t K, int act_mode,
                          int32_t *C, int64_t ldc, const float *scale, const float *bias, float *Cf,
                          int64_t ldcf, void *workspace, size_t workspace_bytes, void *stream);
int fatnn_twobit_gemm_ws(const void *Wp, const void *Ap, int64_t M, int64_t N, int64_t K, int basis,
                         int32_t *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream);
int fatnn_binary_gemm_ws(const void *Wb, const void *Ab, int64_t M, int64_t N, int64_t K, int32_t *C,
                         int64_t ldc, void *workspace, size_t workspace_bytes, void *stream);

/*
 * fatnn_ternary_gemm_ws for callers that cannot allocate device memory and have no workspace to hand in:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * bit-identical results; it always runs the equal-shares schedule, and the scratch memory of that schedule
 * (tile counters and hand-over slots) is a fixed array inside the library, fatnn_noalloc_scratch_bytes()
 * = 64 KiB + 16 MiB on every GPU the library has run this call on, held until the process ends.  The call
 * allocates and frees nothing.
 *   limits   ceil(M/64) * ceil(N/64) <= 16384 tiles (one counter each); beyond that FATNN_ERR_SIZE.
 *   state    every call on one GPU uses that GPU's one array: calls that overlap on a GPU (two streams,
 *            two threads) race and give wrong results; order them.  The call clears what it needs of the
 *            array itself (with a fill kernel, so it may be captured into a HIP graph).
 */
size_t fatnn_noalloc_scratch_bytes(void);
int fatnn_ternary_gemm_noalloc(const void *Wp, const void *Ap, int64_t M, int64_t N, int64_t K, int act_mode,
                               int32_t *C, int64_t ldc, const float *scale, const float *bias, float *Cf,
                               int64_t ldcf, void *stream);

/* FATNN_OK for a zero count of out-of-set inputs, FATNN_ERR_LEVEL otherwise (first constraint of
 * Section 3.3).  `n_invalid_host` is the value of a packing call's counter copied to the host. */
int fatnn_level_status(int64_t n_invalid_host);

/*
 * Measurement switches (no paper passage: they serve the kernel comparisons in the report).
 * Process-wide, stored in atomics, read by every later launch; a negative argument keeps the
 * current value.  Their initial values come from the environment variables FATNN_CONV_KERNEL
 * (=tiled), FATNN_STREAM_WPS, FATNN_STREAM_U7, FATNN_GEMM_EVEN_SHARE and FATNN_GEMM_DEEPK, read once on
 * first use.
 *   conv_kernel         0 = automatic, 1 = convolutions always take the LDS-tiled kernel
 *   stream_wps          wavefronts per SIMD of the column-streaming kernel, 0 = planned, at most 8
 *   seven_pixel_groups  0 = off, 1 = by the size rule, 2 = wherever a kernel exists
 *   gemm_even_share     schedule of the *_gemm_ws calls: 0 = automatic, 1..8 = even shares with that many
 *                       workgroups per compute unit whatever the size, 9 = never, 10 = whole tiles plus a
 *                       split remainder wherever the tile count is not a multiple of the compute units,
 *                       11 = even shares of the small (32 x 32) tile whatever the size
 *   gemm_deepk          kernel for GEMMs with at most 128 columns and K >= 2048 (fully connected layers):
 *                       0 = automatic, 1 = wherever the shape fits, 2 = never
 * Results never depend on these, only the kernel and launch shape chosen.
 */
int fatnn_set_tuning(int conv_kernel, int stream_wps, int seven_pixel_groups, int gemm_even_share, int gemm_deepk);

/*
 * Roofline probes (no paper passage: they measure the denominators of the roofline report on the
 * chip).  Both attach the events of fatnn_time_next_launch to their one kernel.
 *
 * fatnn_probe_valu issues, from registers only, the instruction pair that the reduced form of Eq. 3
 * costs per 32-bit plane word (one three-input logic instruction feeding one accumulating popcount),
 * with `waves_per_simd` wavefronts on every SIMD of the device.
 *   kind            0 pair, all operands in vector registers (as the tiled GEMM kernel issues it)
 *                   1 pair with the data word in a scalar register (as the streaming conv kernel does)
 *                   2 popcount alone   3 logic instruction alone   4 plain two-input xor
 *                   5 pair with its data words re-read from LDS, one 128-bit read per 16 pairs (the large
 *                     GEMM tile's ratio), issued ahead of their use
 *   waves_per_simd  1..8;  iters >= 1 loop iterations of 128 instructions each
 *   scratch         device, 16-byte aligned, at least fatnn_probe_scratch_bytes() bytes; contents
 *                   are read as operand values (any bit pattern) and overwritten
 *   lane_instr      HOST pointer or NULL: receives the number of 32-bit lane-instructions the launch
 *                   executes (workgroups * 256 lanes * iters * 128)
 * fatnn_probe_hbm streams `bytes` (a multiple of 16, below 4 GiB) with 128-bit accesses: kind 0 reads src, 1 writes
 * dst, 2 copies src to dst (bytes read + bytes written = 2 * bytes); the unused pointer may be NULL.
 */
size_t fatnn_probe_scratch_bytes(void);
int fatnn_probe_valu(int kind, int waves_per_simd, int iters, void *scratch, size_t scratch_bytes,
                     int64_t *lane_instr, void *stream);
int fatnn_probe_hbm(int kind, void *dst, const void *src, size_t bytes, void *scratch, size_t scratch_bytes,
                    void *stream);

/*
 * Measurement hook (no paper passage: it serves the roofline report).  The next
 * fatnn_*_gemm / fatnn_*_conv2d / fatnn_probe_* call made by the calling thread attaches the two
 * events to its kernel dispatch, so that hipEventElapsedTime(start, stop) is the
 * duration of that kernel alone, without the launch gap that events recorded around
 * the call would include.  Both are hipEvent_t created by the caller with timing
 * enabled; they stay the caller's.  The hook is consumed by that one launch;
 * (NULL, NULL) clears it.  Giving only one event returns FATNN_ERR_NULL.
 */
int fatnn_time_next_launch(void *start_event, void *stop_event);

const char *fatnn_status_str(int status);
int fatnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FATNN_H */
