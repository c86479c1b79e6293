// Host layer of the C ABI declared in include/fatnn.h: argument checks (all done
// before the first GPU call, so they work with no GPU present), buffer layout, and
// the choice of kernel.  Nothing here computes.
#include "../../include/fatnn.h"
#include "fatnn_device.h"

#include <atomic>
#include <math.h>
#include <stdlib.h>

using namespace fatnn;

namespace fatnn {
namespace {
thread_local LaunchTiming g_timing = {nullptr, nullptr};
}
// The measurement switches: process-wide atomics whose initial values are read from the
// environment exactly once, on first use (the initialisation of a function-local static is
// thread-safe); fatnn_set_tuning overwrites them; launches only read them.
namespace {
struct TuningState {
    std::atomic<int> force_tiled, stream_wps, u7_mode, gemm_even_share, gemm_deepk;
    TuningState() {
        const char* e = getenv("FATNN_CONV_KERNEL");
        force_tiled.store(e != nullptr && e[0] == 't' ? 1 : 0);
        e = getenv("FATNN_STREAM_WPS");
        const int w = e != nullptr ? atoi(e) : 0;
        stream_wps.store(w > 0 ? w : 0);
        e = getenv("FATNN_STREAM_U7");
        u7_mode.store((e != nullptr && e[0] >= '0' && e[0] <= '2') ? e[0] - '0' : 1);
        e = getenv("FATNN_GEMM_EVEN_SHARE");
        const int es = e != nullptr ? atoi(e) : 0;
        gemm_even_share.store(es >= 0 && es <= 11 ? es : 0);
        e = getenv("FATNN_GEMM_DEEPK");
        gemm_deepk.store((e != nullptr && e[0] >= '0' && e[0] <= '2') ? e[0] - '0' : 0);
    }
};
TuningState& tuning_state() {
    static TuningState s;
    return s;
}
}  // namespace
Tuning tuning() {
    TuningState& s = tuning_state();
    Tuning v;
    v.force_tiled = s.force_tiled.load(std::memory_order_relaxed) != 0;
    v.stream_wps = s.stream_wps.load(std::memory_order_relaxed);
    v.u7_mode = s.u7_mode.load(std::memory_order_relaxed);
    v.gemm_even_share = s.gemm_even_share.load(std::memory_order_relaxed);
    v.gemm_deepk = s.gemm_deepk.load(std::memory_order_relaxed);
    return v;
}
void set_tuning(int force_tiled, int stream_wps, int u7_mode, int gemm_even_share, int gemm_deepk) {
    TuningState& s = tuning_state();
    if (force_tiled >= 0) s.force_tiled.store(force_tiled != 0 ? 1 : 0, std::memory_order_relaxed);
    if (stream_wps >= 0) s.stream_wps.store(stream_wps, std::memory_order_relaxed);
    if (u7_mode >= 0) s.u7_mode.store(u7_mode, std::memory_order_relaxed);
    if (gemm_even_share >= 0) s.gemm_even_share.store(gemm_even_share, std::memory_order_relaxed);
    if (gemm_deepk >= 0) s.gemm_deepk.store(gemm_deepk, std::memory_order_relaxed);
}
LaunchTiming take_launch_timing() {
    const LaunchTiming t = g_timing;
    g_timing.start = nullptr;
    g_timing.stop = nullptr;
    return t;
}
}  // namespace fatnn

namespace {

constexpr int64_t kMaxRows = 0x7FFFFFFFLL;

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

struct PackShape {
    int64_t rows, K;
    bool gather;
    GatherDesc g;
};

// Turns (layout, dims) into rows x K plus, for the non-contiguous layouts, the gather rule.
int pack_shape(int layout, const int64_t dims[4], PackShape* out) {
    for (int i = 0; i < 4; ++i)
        if (dims[i] < 0) return FATNN_ERR_SHAPE;
    PackShape s{};
    switch (layout) {
        case FATNN_ROWMAJOR_K:
            s.rows = dims[0];
            s.K = dims[1];
            s.gather = false;
            break;
        case FATNN_NHWC:
        case FATNN_OHWI: {
            const int64_t C = dims[3];
            if (C < 1) return FATNN_ERR_SHAPE;
            if (C % 32 != 0) return FATNN_ERR_UNSUPPORTED;
            if (layout == FATNN_NHWC) {
                if (dims[1] > kMaxRows || dims[2] > kMaxRows) return FATNN_ERR_SIZE;
                if (dims[0] != 0 && dims[1] * dims[2] > kMaxRows / (dims[0] > 0 ? dims[0] : 1)) return FATNN_ERR_SIZE;
                s.rows = dims[0] * dims[1] * dims[2];
                s.K = C;
            } else {
                if (dims[1] < 1 || dims[2] < 1) return FATNN_ERR_SHAPE;
                if (dims[1] > 64 || dims[2] > 64) return FATNN_ERR_SIZE;
                s.rows = dims[0];
                s.K = dims[1] * dims[2] * C;
            }
            s.gather = false;
            break;
        }
        case FATNN_OIHW: {
            const int64_t O = dims[0], C = dims[1], R = dims[2], S = dims[3];
            if (C < 1 || R < 1 || S < 1) return FATNN_ERR_SHAPE;
            if (C % 32 != 0) return FATNN_ERR_UNSUPPORTED;
            if (R > 64 || S > 64) return FATNN_ERR_SIZE;
            s.rows = O;
            s.K = R * S * C;
            s.gather = true;
            // row = o: offset o*C*R*S;  k = (r*S+s)*C + c: offset (r*S+s) + c*R*S
            s.g.n1 = 1; s.g.rs0 = C * R * S; s.g.rs1 = 0;
            s.g.C = C; s.g.ks0 = 1; s.g.ks1 = R * S;
            break;
        }
        case FATNN_NCHW: {
            const int64_t B = dims[0], C = dims[1], H = dims[2], W = dims[3];
            if (C < 1) return FATNN_ERR_SHAPE;
            if (C % 32 != 0) return FATNN_ERR_UNSUPPORTED;
            if (H > kMaxRows || W > kMaxRows) return FATNN_ERR_SIZE;
            if (B != 0 && H * W > kMaxRows / B) return FATNN_ERR_SIZE;
            s.rows = B * H * W;
            s.K = C;
            s.gather = true;
            // row = b*(H*W) + hw: offset b*C*H*W + hw;  k = c: offset c*H*W
            s.g.n1 = (H * W > 0) ? H * W : 1; s.g.rs0 = C * H * W; s.g.rs1 = 1;
            s.g.C = C; s.g.ks0 = 0; s.g.ks1 = H * W;
            break;
        }
        default:
            return FATNN_ERR_UNSUPPORTED;
    }
    if (s.K < 1) return FATNN_ERR_SHAPE;
    if (s.K > FATNN_MAX_K || s.rows > kMaxRows) return FATNN_ERR_SIZE;
    *out = s;
    return FATNN_OK;
}

int pack_common(const int8_t* levels, int layout, const int64_t dims[4], int kind, int role, void* packed,
                size_t packed_bytes, int32_t* n_invalid, void* stream) {
    if (dims == nullptr) return FATNN_ERR_NULL;
    PackShape s;
    int rc = pack_shape(layout, dims, &s);
    if (rc != FATNN_OK) return rc;
    if (s.rows == 0) return FATNN_OK;
    if (levels == nullptr || packed == nullptr) return FATNN_ERR_NULL;
    if (!aligned(packed, 16)) return FATNN_ERR_ALIGN;
    if (n_invalid != nullptr && !aligned(n_invalid, 4)) return FATNN_ERR_ALIGN;
    if (packed_bytes < fatnn_packed_bytes(role, s.rows, s.K)) return FATNN_ERR_SIZE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    plane2* out = reinterpret_cast<plane2*>(packed);
    int lrc = s.gather ? launch_pack_gather(levels, s.rows, s.K, s.g, kind, out, n_invalid, st)
                       : launch_pack_contiguous(levels, s.rows, s.K, kind, out, n_invalid, st);
    if (lrc != 0) return FATNN_ERR_HIP;
    if (role == FATNN_WEIGHT) {
        const int64_t Kw = fatnn_words_per_row(s.K);
        char* base = reinterpret_cast<char*>(packed);
        if (kind == PACK_WEIGHT) {
            int32_t* consts = reinterpret_cast<int32_t*>(base + fatnn_weight_consts_offset(s.rows, s.K));
            if (launch_row_constants(out, s.rows, Kw, consts, consts + s.rows, st) != 0) return FATNN_ERR_HIP;
        }
        plane2* inter = reinterpret_cast<plane2*>(base + fatnn_weight_interleaved_offset(s.rows, s.K));
        if (launch_interleave_weights(out, s.rows, Kw, inter, st) != 0) return FATNN_ERR_HIP;
    }
    return FATNN_OK;
}

int check_gemm_dims(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 1) return FATNN_ERR_SHAPE;
    if (M > kMaxRows || N > kMaxRows || K > FATNN_MAX_K) return FATNN_ERR_SIZE;
    return FATNN_OK;
}

struct ConvShape {
    int64_t Ho, Wo, N, K;
};

int check_conv_dims(int64_t B, int64_t Cin, int64_t H, int64_t W, int64_t Cout, int R, int S, int stride,
                    int pad, ConvShape* cs) {
    if (B < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 0 || R < 1 || S < 1 || stride < 1 || pad < 0)
        return FATNN_ERR_SHAPE;
    if (!(R == S && (R == 1 || R == 3))) return FATNN_ERR_UNSUPPORTED;
    if (!(stride == 1 || stride == 2)) return FATNN_ERR_UNSUPPORTED;
    if (!(pad == 0 || pad == 1) || pad > R / 2) return FATNN_ERR_UNSUPPORTED;
    if (Cin % 32 != 0) return FATNN_ERR_UNSUPPORTED;
    if (H + 2 * pad < R || W + 2 * pad < S) return FATNN_ERR_SHAPE;
    if (H > 65535 || W > 65535 || Cout > kMaxRows) return FATNN_ERR_SIZE;
    cs->Ho = (H + 2 * pad - R) / stride + 1;
    cs->Wo = (W + 2 * pad - S) / stride + 1;
    cs->K = (int64_t)R * S * Cin;
    if (cs->K > FATNN_MAX_K) return FATNN_ERR_SIZE;
    if (B != 0 && cs->Ho * cs->Wo > kMaxRows / B) return FATNN_ERR_SIZE;
    if (B != 0 && H * W > kMaxRows / B) return FATNN_ERR_SIZE;
    cs->N = B * cs->Ho * cs->Wo;
    return FATNN_OK;
}

void set_ternary_consts(GemmParams& p, const void* Wp, int64_t M, int64_t K, int act_mode) {
    const int32_t* consts = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(Wp) +
                                                             fatnn_weight_consts_offset(M, K));
    // symmetric: x.w = nnz - P'.  ReLU: values are one higher, which adds the sum of
    // the weights (npos - nneg): nnz + npos - nneg = 2 * npos.
    if (act_mode == FATNN_RELU) {
        p.rowc = consts + M;
        p.cmul = 2;
    } else {
        p.rowc = consts;
        p.cmul = 1;
    }
}

// Which convolution kernel serves a call.  Tuning::force_tiled overrides the choice (for
// measurements).
bool want_stream(int op, int R, int S, int Cw, int stride) {
    if (!stream_supported(op, R, S, Cw, stride)) return false;
    return !tuning().force_tiled;
}

struct ChainArgs {
    const float* skip;
    int relu;
    float t1, t2;
    uint32_t nan_lo;
    int out_border;
    void* Xnext;
};

int run_conv(const void* Wp, const void* Xp, int x_layout, int64_t B, int64_t Cin, int64_t H, int64_t W,
             int64_t Cout, int R, int S, int stride, int pad, const ConvShape& cs, int op, int act_mode, int32_t* Y,
             const float* scale, const float* bias, float* Yf, void* stream, const ChainArgs* chain = nullptr) {
    const int Cw = (int)(Cin / 32);
    const uint32_t pad_y = (op == OP_TERNARY && act_mode == FATNN_RELU) ? 0u : 0xFFFFFFFFu;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const bool bordered = x_layout != FATNN_X_PLAIN;
    // in the bordered layouts the padding is physical: a larger image convolved without padding
    // (and, when the ring is wider than the padding, with the taps shifted inwards)
    const int xb = x_layout == FATNN_X_BORDERED1 ? 1 : (bordered ? pad : 0);
    const int64_t Hs = H + 2 * xb, Ws = W + 2 * xb;
    const int pad_s = pad - xb;
    const int64_t stored_bytes = (B * Hs * Ws + FATNN_BORDER_SLACK_PIXELS) * Cw * (int64_t)sizeof(plane2);
    // the streaming kernel addresses its input, its outputs and the next layer's buffer with
    // 32-bit byte offsets
    const int64_t out_bytes = cs.N * Cout * 4;
    const int64_t next_bytes =
        chain != nullptr ? (int64_t)fatnn_bordered_act_bytes(B, cs.Ho, cs.Wo, Cout, chain->out_border) : 0;
    if (bordered && stored_bytes < 0xFFFFFFFFLL && out_bytes < 0xFFFFFFFFLL && next_bytes < 0xFFFFFFFFLL &&
        want_stream(op, R, S, Cw, stride)) {
        StreamParams q{};
        q.Wi = reinterpret_cast<const plane2*>(reinterpret_cast<const char*>(Wp) +
                                               fatnn_weight_interleaved_offset(Cout, cs.K));
        q.A = reinterpret_cast<const uint32_t*>(Xp);
        if (op == OP_TERNARY) {
            GemmParams t{};
            set_ternary_consts(t, Wp, Cout, cs.K, act_mode);
            q.rowc = t.rowc;
            q.cmul = t.cmul;
        } else {
            q.cmul = 1;
        }
        q.K = (int32_t)cs.K;
        q.M = (int32_t)Cout;
        q.Kw = (int32_t)(cs.K / 32);
        q.C = Y; q.Cf = Yf; q.ldc = (int32_t)Cout;
        q.out_bytes = (uint32_t)out_bytes;
        q.scale = scale; q.bias = bias;
        q.Hp = (int32_t)Hs; q.Wp = (int32_t)Ws; q.Ho = (int32_t)cs.Ho;
        q.xoff = xb - pad;
        if (chain != nullptr) {
            q.Xn = reinterpret_cast<plane2*>(chain->Xnext);
            q.nborder = chain->out_border;
            q.nHp = (int32_t)(cs.Ho + 2 * chain->out_border);
            q.nWp = (int32_t)(cs.Wo + 2 * chain->out_border);
            q.nCw = (int32_t)(Cout / 32);
            q.skip = chain->skip;
            q.t1 = chain->t1; q.t2 = chain->t2; q.nan_lo = chain->nan_lo;
            q.relu = chain->relu;
        }
        return launch_stream_conv(q, op, R, Cw, stride, B * cs.Ho, cs.Wo, st) == 0 ? FATNN_OK : FATNN_ERR_HIP;
    }
    if (chain != nullptr) return FATNN_ERR_UNSUPPORTED;   // the chaining epilogue lives in the streaming kernel
    GemmParams p{};
    p.W = reinterpret_cast<const plane2*>(Wp);
    p.A = reinterpret_cast<const plane2*>(Xp);
    if (op == OP_TERNARY) set_ternary_consts(p, Wp, Cout, cs.K, act_mode);
    else p.cmul = 1;
    p.K = (int32_t)cs.K;
    p.M = (int32_t)Cout;
    p.N = (int32_t)cs.N;
    p.Kw = (int32_t)(cs.K / 32);
    p.C = Y; p.ldc_m = 1; p.ldc_n = Cout;
    p.Cf = Yf; p.ldf_m = 1; p.ldf_n = Cout;
    p.scale = scale; p.bias = bias;
    p.is_conv = 1;
    p.B = (int32_t)B; p.H = (int32_t)Hs; p.Wd = (int32_t)Ws; p.Cw = Cw;
    p.cw_shift = -1;
    for (int sh = 0; sh < 20; ++sh)
        if ((1 << sh) == Cw) p.cw_shift = sh;
    p.Ho = (int32_t)cs.Ho; p.Wo = (int32_t)cs.Wo; p.R = R; p.S = S; p.stride = stride; p.pad = pad_s;
    // a padded tap is the value 0: level 1 = codec 01 in symmetric mode (and in the two-bit
    // ternary basis), level 0 = codec 00 in ReLU mode
    p.pad_x = 0u;
    p.pad_y = pad_y;
    return launch_gemm(p, op, st) == 0 ? FATNN_OK : FATNN_ERR_HIP;
}

// Level that Eq. 9 (weights, real-valued activations) or Eq. 10 (ReLU activations) gives to p,
// with every operation in float32 and round-half-to-even.
int quantizer_level(float p, bool relu, float a1, float a2) {
    if (!relu) {
        const float neg = nearbyintf(fminf(fmaxf(p / a1, -1.0f), 0.0f));
        const float pos = nearbyintf(fminf(fmaxf(p / a2, 0.0f), 1.0f));
        return (int)(neg + pos) + 1;
    }
    const float first = nearbyintf(fminf(fmaxf(p / a1, 0.0f), 1.0f));
    const float second = nearbyintf(fminf(fmaxf((p - a1) / a2, 0.0f), 1.0f));
    return (int)(first + second);
}

// The quantizer is monotone in p, so "level >= L" holds exactly for p >= some float t.  Starts
// at the real-number threshold and walks to the exact float32 break point.
bool exact_threshold(int L, bool relu, float a1, float a2, float* t_out) {
    float guess;
    if (!relu)
        guess = (L == 1) ? -0.5f * a1 : 0.5f * a2;
    else
        guess = (L == 1) ? 0.5f * a1 : a1 + 0.5f * a2;
    float p = guess;
    for (int it = 0; it < 4096; ++it) {
        if (quantizer_level(p, relu, a1, a2) >= L) {
            const float below = nextafterf(p, -INFINITY);
            if (quantizer_level(below, relu, a1, a2) < L) {
                *t_out = p;
                return true;
            }
            p = below;
        } else {
            p = nextafterf(p, INFINITY);
        }
    }
    return false;
}

int quant_setup(int role, int act_mode, float alpha1, float alpha2, float* t1, float* t2, uint32_t* nan_lo) {
    if (role != FATNN_WEIGHT && role != FATNN_ACT) return FATNN_ERR_UNSUPPORTED;
    if (act_mode != FATNN_SYM && act_mode != FATNN_RELU) return FATNN_ERR_UNSUPPORTED;
    if (!(alpha1 > 0.0f) || !(alpha2 > 0.0f) || !isfinite(alpha1) || !isfinite(alpha2)) return FATNN_ERR_SHAPE;
    const bool relu = role == FATNN_ACT && act_mode == FATNN_RELU;
    if (!exact_threshold(1, relu, alpha1, alpha2, t1) || !exact_threshold(2, relu, alpha1, alpha2, t2))
        return FATNN_ERR_UNSUPPORTED;
    // A NaN is outside the quantizers' domain: it is packed as the VALUE 0 (and counted where the call
    // has a counter).  Value 0 is level 1 = planes (0, 1) for weights and symmetric activations, level 0
    // = planes (0, 0) for ReLU-mode activations; both comparisons are false for a NaN, so only the low
    // plane bit needs to be supplied.
    *nan_lo = relu ? 0u : 1u;
    return FATNN_OK;
}

int pack_bordered_common(const int8_t* levels, const int64_t dims[4], int border, int kind, plane2 border_word,
                         void* packed, size_t packed_bytes, int32_t* n_invalid, void* stream) {
    if (dims == nullptr) return FATNN_ERR_NULL;
    const int64_t B = dims[0], H = dims[1], W = dims[2], C = dims[3];
    if (B < 0 || H < 1 || W < 1 || C < 1) return FATNN_ERR_SHAPE;
    if (border < 0 || border > 1) return FATNN_ERR_UNSUPPORTED;
    if (C % 32 != 0) return FATNN_ERR_UNSUPPORTED;
    if (H > 65535 || W > 65535 || C > FATNN_MAX_K) return FATNN_ERR_SIZE;
    if (B != 0 && (H + 2) * (W + 2) > kMaxRows / B) return FATNN_ERR_SIZE;
    if (levels == nullptr && B > 0) return FATNN_ERR_NULL;
    if (packed == nullptr) return FATNN_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(levels, 16) || !aligned(n_invalid, 4)) return FATNN_ERR_ALIGN;
    if (packed_bytes < fatnn_bordered_act_bytes(B, H, W, C, border)) return FATNN_ERR_SIZE;
    return launch_pack_bordered(levels, B, H, W, C, border, kind, border_word, FATNN_BORDER_SLACK_PIXELS,
                                reinterpret_cast<plane2*>(packed), n_invalid,
                                reinterpret_cast<hipStream_t>(stream)) == 0
               ? FATNN_OK
               : FATNN_ERR_HIP;
}

}  // namespace

extern "C" {

int64_t fatnn_words_per_row(int64_t K) { return K < 1 ? -1 : (K + 31) / 32; }

size_t fatnn_weight_consts_offset(int64_t rows, int64_t K) {
    if (rows < 0 || K < 1) return 0;
    return round_up((size_t)rows * (size_t)fatnn_words_per_row(K) * sizeof(plane2), 256);
}

size_t fatnn_packed_bytes(int role, int64_t rows, int64_t K) {
    if (rows < 0 || K < 1 || (role != FATNN_WEIGHT && role != FATNN_ACT)) return 0;
    const size_t words = (size_t)rows * (size_t)fatnn_words_per_row(K) * sizeof(plane2);
    if (role == FATNN_ACT) return words;
    return fatnn_weight_interleaved_offset(rows, K) +
           (size_t)((rows + 63) / 64) * 64 * (size_t)fatnn_words_per_row(K) * sizeof(plane2);
}

size_t fatnn_weight_interleaved_offset(int64_t rows, int64_t K) {
    if (rows < 0 || K < 1) return 0;
    return fatnn_weight_consts_offset(rows, K) + round_up((size_t)rows * 2 * sizeof(int32_t), 256);
}

int fatnn_pack_ternary(const int8_t* levels, int layout, const int64_t dims[4], int role, void* packed,
                       size_t packed_bytes, int32_t* n_invalid, void* stream) {
    if (role != FATNN_WEIGHT && role != FATNN_ACT) return FATNN_ERR_UNSUPPORTED;
    return pack_common(levels, layout, dims, role == FATNN_WEIGHT ? PACK_WEIGHT : PACK_ACT, role, packed,
                       packed_bytes, n_invalid, stream);
}

int fatnn_pack_twobit(const int8_t* codes, int layout, const int64_t dims[4], int role, void* packed,
                      size_t packed_bytes, int32_t* n_invalid, void* stream) {
    if (role != FATNN_WEIGHT && role != FATNN_ACT) return FATNN_ERR_UNSUPPORTED;
    return pack_common(codes, layout, dims, PACK_TWOBIT, role, packed, packed_bytes, n_invalid, stream);
}

int fatnn_quantize_pack(const float* x, int layout, const int64_t dims[4], int role, int act_mode, float alpha1,
                        float alpha2, void* packed, size_t packed_bytes, int32_t* n_invalid, void* stream) {
    if (dims == nullptr) return FATNN_ERR_NULL;
    if (layout != FATNN_ROWMAJOR_K && layout != FATNN_NHWC && layout != FATNN_OHWI) return FATNN_ERR_UNSUPPORTED;
    PackShape s;
    int rc = pack_shape(layout, dims, &s);
    if (rc != FATNN_OK) return rc;
    float t1, t2;
    uint32_t nan_lo;
    rc = quant_setup(role, act_mode, alpha1, alpha2, &t1, &t2, &nan_lo);
    if (rc != FATNN_OK) return rc;
    if (s.rows == 0) return FATNN_OK;
    if (x == nullptr || packed == nullptr) return FATNN_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(x, 4) || !aligned(n_invalid, 4)) return FATNN_ERR_ALIGN;
    if (packed_bytes < fatnn_packed_bytes(role, s.rows, s.K)) return FATNN_ERR_SIZE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    plane2* out = reinterpret_cast<plane2*>(packed);
    if (launch_quantize_pack(x, s.rows, s.K, role == FATNN_WEIGHT ? PACK_WEIGHT : PACK_ACT, t1, t2, nan_lo, out,
                             n_invalid, st) != 0)
        return FATNN_ERR_HIP;
    if (role == FATNN_WEIGHT) {
        const int64_t Kw = fatnn_words_per_row(s.K);
        char* base = reinterpret_cast<char*>(packed);
        int32_t* consts = reinterpret_cast<int32_t*>(base + fatnn_weight_consts_offset(s.rows, s.K));
        if (launch_row_constants(out, s.rows, Kw, consts, consts + s.rows, st) != 0) return FATNN_ERR_HIP;
        plane2* inter = reinterpret_cast<plane2*>(base + fatnn_weight_interleaved_offset(s.rows, s.K));
        if (launch_interleave_weights(out, s.rows, Kw, inter, st) != 0) return FATNN_ERR_HIP;
    }
    return FATNN_OK;
}

int fatnn_quantize_pack_bordered(const float* x, const int64_t dims[4], int border, int act_mode, float alpha1,
                                 float alpha2, void* packed, size_t packed_bytes, int32_t* n_invalid, void* stream) {
    if (dims == nullptr) return FATNN_ERR_NULL;
    const int64_t B = dims[0], H = dims[1], W = dims[2], C = dims[3];
    if (B < 0 || H < 1 || W < 1 || C < 1) return FATNN_ERR_SHAPE;
    if (border < 0 || border > 1) return FATNN_ERR_UNSUPPORTED;
    if (C % 32 != 0) return FATNN_ERR_UNSUPPORTED;
    if (H > 65535 || W > 65535 || C > FATNN_MAX_K) return FATNN_ERR_SIZE;
    if (B != 0 && (H + 2) * (W + 2) > kMaxRows / B) return FATNN_ERR_SIZE;
    float t1, t2;
    uint32_t nan_lo;
    int rc = quant_setup(FATNN_ACT, act_mode, alpha1, alpha2, &t1, &t2, &nan_lo);
    if (rc != FATNN_OK) return rc;
    if (x == nullptr && B > 0) return FATNN_ERR_NULL;
    if (packed == nullptr) return FATNN_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(x, 16) || !aligned(n_invalid, 4)) return FATNN_ERR_ALIGN;
    if (packed_bytes < fatnn_bordered_act_bytes(B, H, W, C, border)) return FATNN_ERR_SIZE;
    plane2 bw;
    bw.x = 0u;
    bw.y = act_mode == FATNN_SYM ? 0xFFFFFFFFu : 0u;
    return launch_quantize_pack_bordered(x, B, H, W, C, border, bw, FATNN_BORDER_SLACK_PIXELS, t1, t2, nan_lo,
                                         reinterpret_cast<plane2*>(packed), n_invalid,
                                         reinterpret_cast<hipStream_t>(stream)) == 0
               ? FATNN_OK
               : FATNN_ERR_HIP;
}

int fatnn_ternary_gemm(const void* Wp, const void* Ap, int64_t M, int64_t N, int64_t K, int act_mode,
                       int32_t* C, int64_t ldc, const float* scale, const float* bias, float* Cf,
                       int64_t ldcf, void* stream) {
    return fatnn_ternary_gemm_ws(Wp, Ap, M, N, K, act_mode, C, ldc, scale, bias, Cf, ldcf, nullptr, 0, stream);
}

int fatnn_ternary_gemm_ws(const void* Wp, const void* Ap, int64_t M, int64_t N, int64_t K, int act_mode,
                          int32_t* C, int64_t ldc, const float* scale, const float* bias, float* Cf,
                          int64_t ldcf, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_gemm_dims(M, N, K);
    if (rc != FATNN_OK) return rc;
    if (act_mode != FATNN_SYM && act_mode != FATNN_RELU) return FATNN_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return FATNN_OK;   // nothing to compute: output pointers may be null
    if (C == nullptr && Cf == nullptr) return FATNN_ERR_NULL;
    if (Cf != nullptr && scale == nullptr) return FATNN_ERR_NULL;
    if (C != nullptr && ldc < N) return FATNN_ERR_SHAPE;
    if (Cf != nullptr && ldcf < N) return FATNN_ERR_SHAPE;
    if (Wp == nullptr || Ap == nullptr) return FATNN_ERR_NULL;
    if (!aligned(Wp, 16) || !aligned(Ap, 16) || !aligned(C, 4) || !aligned(Cf, 4) || !aligned(scale, 4) ||
        !aligned(bias, 4) || !aligned(workspace, 16))
        return FATNN_ERR_ALIGN;
    GemmParams p{};
    p.ws = workspace;
    p.ws_bytes = workspace != nullptr ? workspace_bytes : 0;
    p.W = reinterpret_cast<const plane2*>(Wp);
    p.A = reinterpret_cast<const plane2*>(Ap);
    set_ternary_consts(p, Wp, M, K, act_mode);
    p.K = (int32_t)K;
    p.M = (int32_t)M;
    p.N = (int32_t)N;
    p.Kw = (int32_t)fatnn_words_per_row(K);
    p.C = C; p.ldc_m = ldc; p.ldc_n = 1;
    p.Cf = Cf; p.ldf_m = ldcf; p.ldf_n = 1;
    p.scale = scale; p.bias = bias;
    p.is_conv = 0;
    return launch_gemm(p, OP_TERNARY, reinterpret_cast<hipStream_t>(stream)) == 0 ? FATNN_OK : FATNN_ERR_HIP;
}

size_t fatnn_bordered_act_bytes(int64_t B, int64_t H, int64_t W, int64_t C, int border) {
    if (B < 0 || H < 1 || W < 1 || C < 1 || C % 32 != 0 || border < 0 || border > 1) return 0;
    return (size_t)(B * (H + 2 * border) * (W + 2 * border) + FATNN_BORDER_SLACK_PIXELS) * (size_t)(C / 32) *
           sizeof(plane2);
}

int fatnn_pack_ternary_bordered(const int8_t* levels, const int64_t dims[4], int border, int act_mode, void* packed,
                                size_t packed_bytes, int32_t* n_invalid, void* stream) {
    if (act_mode != FATNN_SYM && act_mode != FATNN_RELU) return FATNN_ERR_UNSUPPORTED;
    plane2 bw;
    bw.x = 0u;
    bw.y = act_mode == FATNN_SYM ? 0xFFFFFFFFu : 0u;   // level 1 = codec 01  |  level 0 = codec 00
    return pack_bordered_common(levels, dims, border, PACK_ACT, bw, packed, packed_bytes, n_invalid, stream);
}

int fatnn_pack_twobit_bordered(const int8_t* codes, const int64_t dims[4], int border, void* packed,
                               size_t packed_bytes, int32_t* n_invalid, void* stream) {
    plane2 bw;
    bw.x = 0u;
    bw.y = 0xFFFFFFFFu;   // code 01
    return pack_bordered_common(codes, dims, border, PACK_TWOBIT, bw, packed, packed_bytes, n_invalid, stream);
}

int fatnn_ternary_conv2d(const void* Wp, const void* Xp, int x_layout, int64_t B, int64_t Cin, int64_t H,
                         int64_t W, int64_t Cout, int R, int S, int stride, int pad, int act_mode, int32_t* Y,
                         const float* scale, const float* bias, float* Yf, void* stream) {
    if (x_layout != FATNN_X_PLAIN && x_layout != FATNN_X_BORDERED && x_layout != FATNN_X_BORDERED1)
        return FATNN_ERR_UNSUPPORTED;
    ConvShape cs;
    int rc = check_conv_dims(B, Cin, H, W, Cout, R, S, stride, pad, &cs);
    if (rc != FATNN_OK) return rc;
    if (act_mode != FATNN_SYM && act_mode != FATNN_RELU) return FATNN_ERR_UNSUPPORTED;
    if (B == 0 || Cout == 0) return FATNN_OK;
    if (Y == nullptr && Yf == nullptr) return FATNN_ERR_NULL;
    if (Yf != nullptr && scale == nullptr) return FATNN_ERR_NULL;
    if (Wp == nullptr || Xp == nullptr) return FATNN_ERR_NULL;
    if (!aligned(Wp, 16) || !aligned(Xp, 16) || !aligned(Y, 4) || !aligned(Yf, 4) || !aligned(scale, 4) ||
        !aligned(bias, 4))
        return FATNN_ERR_ALIGN;
    return run_conv(Wp, Xp, x_layout, B, Cin, H, W, Cout, R, S, stride, pad, cs, OP_TERNARY, act_mode, Y, scale,
                    bias, Yf, stream);
}

int fatnn_bordered_act_init(void* packed, size_t packed_bytes, int64_t B, int64_t H, int64_t W, int64_t C, int border,
                            int act_mode, void* stream) {
    if (act_mode != FATNN_SYM && act_mode != FATNN_RELU) return FATNN_ERR_UNSUPPORTED;
    const size_t need = fatnn_bordered_act_bytes(B, H, W, C, border);
    if (need == 0) return (border < 0 || border > 1 || (C > 0 && C % 32 != 0)) ? FATNN_ERR_UNSUPPORTED : FATNN_ERR_SHAPE;
    if (packed == nullptr) return FATNN_ERR_NULL;
    if (!aligned(packed, 16)) return FATNN_ERR_ALIGN;
    if (packed_bytes < need) return FATNN_ERR_SIZE;
    plane2 bw;
    bw.x = 0u;
    bw.y = act_mode == FATNN_SYM ? 0xFFFFFFFFu : 0u;
    return launch_fill_words(reinterpret_cast<plane2*>(packed), (int64_t)(need / sizeof(plane2)), bw,
                             reinterpret_cast<hipStream_t>(stream)) == 0
               ? FATNN_OK
               : FATNN_ERR_HIP;
}

int fatnn_ternary_conv2d_chain(const void* Wp, const void* Xp, int x_layout, int64_t B, int64_t Cin, int64_t H,
                               int64_t W, int64_t Cout, int R, int S, int stride, int pad, int act_mode, const float* scale,
                               const float* bias, const float* skip, int relu, float alpha1, float alpha2,
                               int out_act_mode, int out_border, void* Xnext, size_t xnext_bytes, float* Yf,
                               void* stream) {
    if (x_layout != FATNN_X_BORDERED && x_layout != FATNN_X_BORDERED1) return FATNN_ERR_UNSUPPORTED;
    ConvShape cs;
    int rc = check_conv_dims(B, Cin, H, W, Cout, R, S, stride, pad, &cs);
    if (rc != FATNN_OK) return rc;
    if (act_mode != FATNN_SYM && act_mode != FATNN_RELU) return FATNN_ERR_UNSUPPORTED;
    if (out_border < 0 || out_border > 1) return FATNN_ERR_UNSUPPORTED;
    if (Cout % 32 != 0) return FATNN_ERR_UNSUPPORTED;
    if (!stream_supported(OP_TERNARY, R, S, (int)(Cin / 32), stride)) return FATNN_ERR_UNSUPPORTED;
    ChainArgs ch{};
    rc = quant_setup(FATNN_ACT, out_act_mode, alpha1, alpha2, &ch.t1, &ch.t2, &ch.nan_lo);
    if (rc != FATNN_OK) return rc;
    if (B == 0 || Cout == 0) return FATNN_OK;
    if (Wp == nullptr || Xp == nullptr || scale == nullptr || Xnext == nullptr) return FATNN_ERR_NULL;
    if (!aligned(Wp, 16) || !aligned(Xp, 16) || !aligned(Xnext, 16) || !aligned(Yf, 4) || !aligned(scale, 4) ||
        !aligned(bias, 4) || !aligned(skip, 4))
        return FATNN_ERR_ALIGN;
    if (xnext_bytes < fatnn_bordered_act_bytes(B, cs.Ho, cs.Wo, Cout, out_border)) return FATNN_ERR_SIZE;
    ch.skip = skip;
    ch.relu = relu != 0;
    ch.out_border = out_border;
    ch.Xnext = Xnext;
    return run_conv(Wp, Xp, x_layout, B, Cin, H, W, Cout, R, S, stride, pad, cs, OP_TERNARY, act_mode, nullptr, scale,
                    bias, Yf, stream, &ch);
}

// ---- the entry point that allocates nothing -------------------------------------------------------------
// Scratch of the even-share schedule in a file-scope device array: tile counters followed by two hand-over
// slots (64 x 64 int32 each) for 512 workgroups.  Every GPU the library runs on holds its own copy until
// the process ends.  The array's name is a host-side stand-in; the device address is asked for once per
// device (with that device current) and only that address is ever handed to a launch.
namespace {
constexpr int kNoAllocWorkgroups = 512;
constexpr size_t kNoAllocScratchBytes = (size_t)kEvenShareCounterBytes + (size_t)kNoAllocWorkgroups * 2 * (64 * 64 * 4);
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int scratch_for_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FATNN_ERR_HIP;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return FATNN_ERR_HIP;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // concurrent first calls store the same address
    }
    *out = ptr;
    return FATNN_OK;
}
}  // namespace

size_t fatnn_noalloc_scratch_bytes(void) { return kNoAllocScratchBytes; }

int fatnn_ternary_gemm_noalloc(const void* Wp, const void* Ap, int64_t M, int64_t N, int64_t K, int act_mode,
                               int32_t* C, int64_t ldc, const float* scale, const float* bias, float* Cf,
                               int64_t ldcf, void* stream) {
    int rc = check_gemm_dims(M, N, K);
    if (rc != FATNN_OK) return rc;
    if (act_mode != FATNN_SYM && act_mode != FATNN_RELU) return FATNN_ERR_UNSUPPORTED;
    // the scratch has one counter per 64 x 64 tile
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64);
    const int64_t stages = (fatnn_words_per_row(K) + 7) / 8;
    if (tiles > kEvenShareCounterBytes / 4 || tiles * stages >= 0x7FFFFFFFLL) return FATNN_ERR_SIZE;
    if (M == 0 || N == 0) return FATNN_OK;
    if (C == nullptr && Cf == nullptr) return FATNN_ERR_NULL;
    if (Cf != nullptr && scale == nullptr) return FATNN_ERR_NULL;
    if (C != nullptr && ldc < N) return FATNN_ERR_SHAPE;
    if (Cf != nullptr && ldcf < N) return FATNN_ERR_SHAPE;
    if (Wp == nullptr || Ap == nullptr) return FATNN_ERR_NULL;
    if (!aligned(Wp, 16) || !aligned(Ap, 16) || !aligned(C, 4) || !aligned(Cf, 4) || !aligned(scale, 4) ||
        !aligned(bias, 4))
        return FATNN_ERR_ALIGN;
    void* ptr = nullptr;
    rc = scratch_for_current_device(&ptr);
    if (rc != FATNN_OK) return rc;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // The array keeps what the last call left.  A completed call leaves the counters at zero, but a call
    // must not depend on that: the counters of this call's tiles are cleared first, with a fill kernel
    // (which, unlike a memset node, is safe inside a captured graph).
    plane2 zero;
    zero.x = 0u;
    zero.y = 0u;
    if (launch_fill_words(reinterpret_cast<plane2*>(ptr), (tiles * 4 + 7) / 8, zero, st) != 0) return FATNN_ERR_HIP;
    GemmParams p{};
    p.ws = ptr;
    p.ws_bytes = kNoAllocScratchBytes;
    p.W = reinterpret_cast<const plane2*>(Wp);
    p.A = reinterpret_cast<const plane2*>(Ap);
    set_ternary_consts(p, Wp, M, K, act_mode);
    p.K = (int32_t)K;
    p.M = (int32_t)M;
    p.N = (int32_t)N;
    p.Kw = (int32_t)fatnn_words_per_row(K);
    p.C = C; p.ldc_m = ldc; p.ldc_n = 1;
    p.Cf = Cf; p.ldf_m = ldcf; p.ldf_n = 1;
    p.scale = scale; p.bias = bias;
    p.is_conv = 0;
    return launch_ternary_gemm_even_share(p, 2, st) == 0 ? FATNN_OK : FATNN_ERR_HIP;
}

int fatnn_twobit_gemm(const void* Wp, const void* Ap, int64_t M, int64_t N, int64_t K, int basis, int32_t* C,
                      int64_t ldc, void* stream) {
    return fatnn_twobit_gemm_ws(Wp, Ap, M, N, K, basis, C, ldc, nullptr, 0, stream);
}

int fatnn_twobit_gemm_ws(const void* Wp, const void* Ap, int64_t M, int64_t N, int64_t K, int basis, int32_t* C,
                         int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_gemm_dims(M, N, K);
    if (rc != FATNN_OK) return rc;
    if (basis != FATNN_BASIS_TERNARY && basis != FATNN_BASIS_UNIFORM && basis != FATNN_BASIS_XNOR_ONLY)
        return FATNN_ERR_UNSUPPORTED;
    if (basis == FATNN_BASIS_UNIFORM && K > (1 << 20)) return FATNN_ERR_SIZE;   // |C| <= 9K in int32
    if (M == 0 || N == 0) return FATNN_OK;
    if (C == nullptr) return FATNN_ERR_NULL;
    if (ldc < N) return FATNN_ERR_SHAPE;
    if (Wp == nullptr || Ap == nullptr) return FATNN_ERR_NULL;
    if (!aligned(Wp, 16) || !aligned(Ap, 16) || !aligned(C, 4) || !aligned(workspace, 16)) return FATNN_ERR_ALIGN;
    GemmParams p{};
    p.ws = workspace;
    p.ws_bytes = workspace != nullptr ? workspace_bytes : 0;
    p.W = reinterpret_cast<const plane2*>(Wp);
    p.A = reinterpret_cast<const plane2*>(Ap);
    p.K = (int32_t)K;
    p.M = (int32_t)M;
    p.N = (int32_t)N;
    p.Kw = (int32_t)fatnn_words_per_row(K);
    p.C = C; p.ldc_m = ldc; p.ldc_n = 1;
    p.is_conv = 0;
    const int op = basis == FATNN_BASIS_TERNARY ? OP_TWOBIT_TERNARY
                                                : (basis == FATNN_BASIS_UNIFORM ? OP_TWOBIT_UNIFORM : OP_XOR_PAIR);
    p.cmul = 1;   // xnor rule on codecs: K - popcount(xor)
    return launch_gemm(p, op, reinterpret_cast<hipStream_t>(stream)) == 0 ? FATNN_OK : FATNN_ERR_HIP;
}

int fatnn_twobit_conv2d(const void* Wp, const void* Xp, int x_layout, int64_t B, int64_t Cin, int64_t H,
                        int64_t W, int64_t Cout, int R, int S, int stride, int pad, int basis, int32_t* Y,
                        void* stream) {
    if (x_layout != FATNN_X_PLAIN && x_layout != FATNN_X_BORDERED && x_layout != FATNN_X_BORDERED1)
        return FATNN_ERR_UNSUPPORTED;
    ConvShape cs;
    int rc = check_conv_dims(B, Cin, H, W, Cout, R, S, stride, pad, &cs);
    if (rc != FATNN_OK) return rc;
    if (basis != FATNN_BASIS_TERNARY && basis != FATNN_BASIS_XNOR_ONLY) return FATNN_ERR_UNSUPPORTED;
    if (B == 0 || Cout == 0) return FATNN_OK;
    if (Y == nullptr) return FATNN_ERR_NULL;
    if (Wp == nullptr || Xp == nullptr) return FATNN_ERR_NULL;
    if (!aligned(Wp, 16) || !aligned(Xp, 16) || !aligned(Y, 4)) return FATNN_ERR_ALIGN;
    return run_conv(Wp, Xp, x_layout, B, Cin, H, W, Cout, R, S, stride, pad, cs,
                    basis == FATNN_BASIS_TERNARY ? OP_TWOBIT_TERNARY : OP_XOR_PAIR, FATNN_SYM, Y, nullptr, nullptr,
                    nullptr, stream);
}

// seed words + one result word per thread of the largest probe grid (8 wavefronts per SIMD on up to 1024 CUs)
static constexpr size_t kProbeSeedBytes = 4096;
static constexpr int kProbeMaxCUs = 1024;
size_t fatnn_probe_scratch_bytes(void) { return kProbeSeedBytes + (size_t)kProbeMaxCUs * 8 * 256 * 4; }

static int probe_cu_count(int* cus) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return FATNN_ERR_HIP;
    if (prop.multiProcessorCount < 1 || prop.multiProcessorCount > kProbeMaxCUs) return FATNN_ERR_UNSUPPORTED;
    *cus = prop.multiProcessorCount;
    return FATNN_OK;
}

int fatnn_probe_valu(int kind, int waves_per_simd, int iters, void* scratch, size_t scratch_bytes,
                     int64_t* lane_instr, void* stream) {
    if (kind < 0 || kind > 5) return FATNN_ERR_UNSUPPORTED;
    if (waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) return FATNN_ERR_SHAPE;
    if (scratch == nullptr) return FATNN_ERR_NULL;
    if (!aligned(scratch, 16)) return FATNN_ERR_ALIGN;
    if (scratch_bytes < fatnn_probe_scratch_bytes()) return FATNN_ERR_SIZE;
    int cus = 0;
    const int rc = probe_cu_count(&cus);
    if (rc != FATNN_OK) return rc;
    // one workgroup = four wavefronts = one per SIMD of the CU it lands on
    const int blocks = cus * waves_per_simd;
    if (lane_instr != nullptr)
        *lane_instr = (int64_t)blocks * 256 * iters * probe_pairs_per_iteration() * 2;
    char* base = reinterpret_cast<char*>(scratch);
    return launch_valu_probe(kind, blocks, iters, reinterpret_cast<const uint32_t*>(base),
                             reinterpret_cast<int32_t*>(base + kProbeSeedBytes),
                             reinterpret_cast<hipStream_t>(stream)) == 0
               ? FATNN_OK
               : FATNN_ERR_HIP;
}

int fatnn_probe_hbm(int kind, void* dst, const void* src, size_t bytes, void* scratch, size_t scratch_bytes,
                    void* stream) {
    if (kind < 0 || kind > 2) return FATNN_ERR_UNSUPPORTED;
    if (bytes == 0 || bytes % 16 != 0) return FATNN_ERR_SHAPE;
    if (bytes > 0xFFFFFFF0ull) return FATNN_ERR_SIZE;   // 32-bit buffer offsets
    if ((kind != 1 && src == nullptr) || (kind != 0 && dst == nullptr) || scratch == nullptr) return FATNN_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16) || !aligned(scratch, 16)) return FATNN_ERR_ALIGN;
    if (scratch_bytes < fatnn_probe_scratch_bytes()) return FATNN_ERR_SIZE;
    int cus = 0;
    const int rc = probe_cu_count(&cus);
    if (rc != FATNN_OK) return rc;
    return launch_hbm_probe(kind, dst, src, bytes, cus * 8,
                            reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(scratch) + kProbeSeedBytes),
                            reinterpret_cast<hipStream_t>(stream)) == 0
               ? FATNN_OK
               : FATNN_ERR_HIP;
}

int fatnn_level_status(int64_t n_invalid_host) { return n_invalid_host == 0 ? FATNN_OK : FATNN_ERR_LEVEL; }

int fatnn_set_tuning(int conv_kernel, int stream_wps, int seven_pixel_groups, int gemm_even_share, int gemm_deepk) {
    if (conv_kernel > 1 || stream_wps > 8 || seven_pixel_groups > 2 || gemm_even_share > 11 || gemm_deepk > 2)
        return FATNN_ERR_UNSUPPORTED;
    fatnn::set_tuning(conv_kernel, stream_wps, seven_pixel_groups, gemm_even_share, gemm_deepk);
    return FATNN_OK;
}

int fatnn_time_next_launch(void* start_event, void* stop_event) {
    if ((start_event == nullptr) != (stop_event == nullptr)) return FATNN_ERR_NULL;
    fatnn::g_timing.start = reinterpret_cast<hipEvent_t>(start_event);
    fatnn::g_timing.stop = reinterpret_cast<hipEvent_t>(stop_event);
    return FATNN_OK;
}

int fatnn_pack_binary(const int8_t* bits, int64_t rows, int64_t K, void* packed, size_t packed_bytes,
                      int32_t* n_invalid, void* stream) {
    if (rows < 0 || K < 1) return FATNN_ERR_SHAPE;
    if (rows > kMaxRows || K > 2 * (int64_t)FATNN_MAX_K) return FATNN_ERR_SIZE;
    if (rows == 0) return FATNN_OK;
    if (bits == nullptr || packed == nullptr) return FATNN_ERR_NULL;
    if (!aligned(packed, 16) || !aligned(n_invalid, 4)) return FATNN_ERR_ALIGN;
    if (packed_bytes < fatnn_binary_packed_bytes(rows, K)) return FATNN_ERR_SIZE;
    return launch_pack_binary(bits, rows, K, reinterpret_cast<plane2*>(packed), n_invalid,
                              reinterpret_cast<hipStream_t>(stream)) == 0
               ? FATNN_OK
               : FATNN_ERR_HIP;
}

size_t fatnn_binary_packed_bytes(int64_t rows, int64_t K) {
    if (rows < 0 || K < 1) return 0;
    return (size_t)rows * (size_t)((K + 63) / 64) * sizeof(plane2);
}

int fatnn_binary_gemm(const void* Wb, const void* Ab, int64_t M, int64_t N, int64_t K, int32_t* C, int64_t ldc,
                      void* stream) {
    return fatnn_binary_gemm_ws(Wb, Ab, M, N, K, C, ldc, nullptr, 0, stream);
}

size_t fatnn_gemm_workspace_bytes(void) {
    // tile counters + two hand-over slots for each of 4 workgroups per compute unit on 256 compute units,
    // sized for the largest tile accumulator set (64 x 32 outputs of three words in the uniform two-bit basis)
    return (size_t)kEvenShareCounterBytes + (size_t)1024 * 2 * (64 * 32 * 3 * 4);
}

int fatnn_gemm_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (workspace == nullptr) return FATNN_ERR_NULL;
    if (!aligned(workspace, 16)) return FATNN_ERR_ALIGN;
    if (workspace_bytes < (size_t)kEvenShareCounterBytes) return FATNN_ERR_SIZE;
    plane2 zero;
    zero.x = 0u;
    zero.y = 0u;
    return launch_fill_words(reinterpret_cast<plane2*>(workspace), (int64_t)(workspace_bytes / sizeof(plane2)),
                             zero, reinterpret_cast<hipStream_t>(stream)) == 0
               ? FATNN_OK
               : FATNN_ERR_HIP;
}

int fatnn_binary_gemm_ws(const void* Wb, const void* Ab, int64_t M, int64_t N, int64_t K, int32_t* C, int64_t ldc,
                         void* workspace, size_t workspace_bytes, void* stream) {
    if (M < 0 || N < 0 || K < 1) return FATNN_ERR_SHAPE;
    if (M > kMaxRows || N > kMaxRows || K > 2 * (int64_t)FATNN_MAX_K) return FATNN_ERR_SIZE;
    if (M == 0 || N == 0) return FATNN_OK;
    if (C == nullptr || Wb == nullptr || Ab == nullptr) return FATNN_ERR_NULL;
    if (ldc < N) return FATNN_ERR_SHAPE;
    if (!aligned(Wb, 16) || !aligned(Ab, 16) || !aligned(C, 4) || !aligned(workspace, 16)) return FATNN_ERR_ALIGN;
    GemmParams p{};
    p.ws = workspace;
    p.ws_bytes = workspace != nullptr ? workspace_bytes : 0;
    p.W = reinterpret_cast<const plane2*>(Wb);
    p.A = reinterpret_cast<const plane2*>(Ab);
    p.K = (int32_t)K;
    p.cmul = 2;   // Eq. 1: 2 * popcount(xnor) - N = N - 2 * popcount(xor)
    p.M = (int32_t)M;
    p.N = (int32_t)N;
    p.Kw = (int32_t)((K + 63) / 64);
    p.C = C; p.ldc_m = ldc; p.ldc_n = 1;
    p.is_conv = 0;
    return launch_gemm(p, OP_XOR_PAIR, reinterpret_cast<hipStream_t>(stream)) == 0 ? FATNN_OK : FATNN_ERR_HIP;
}

const char* fatnn_status_str(int status) {
    switch (status) {
        case FATNN_OK: return "ok";
        case FATNN_ERR_NULL: return "required pointer is null";
        case FATNN_ERR_SHAPE: return "invalid or inconsistent dimensions";
        case FATNN_ERR_LEVEL: return "level outside {0,1,2}";
        case FATNN_ERR_ALIGN: return "pointer not aligned as required";
        case FATNN_ERR_SIZE: return "buffer too small or dimension beyond the supported range";
        case FATNN_ERR_UNSUPPORTED: return "configuration not supported";
        case FATNN_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int fatnn_version(void) { return 100; }

}  // extern "C"
