// C-ABI entry points, the host-side plan builder (arch -> fixed list of kernel launches) and the
// weight re-layout into MFMA fragment order.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "accerl_internal.h"

using namespace accerl;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

}  // namespace

// error reporting for the other translation units of the C ABI
int accerl::set_error(int code, const char* msg) {
    g_err = msg;
    return code;
}

namespace {

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(ACCERL_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

inline int64_t up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline int out_hw(int h, int k, int s, int p) { return (h + 2 * p - k) / s + 1; }

uint16_t host_bf16(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)(u >> 16);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ------------------------------------------------------------------ blob layout
enum WType { W_I8, W_F32 };
struct TensorSpec {
    int layer;        // arch layer index; n_layers = heads
    int sub;          // 0: conv/dense/convA/lstm_ih, 1: convB / lstm_hh
    int64_t rows, cols;   // W is [rows, cols]
    bool has_bias;
    WType wt;
    int64_t w_off, b_off; // byte offsets in the weight blob
    int64_t sw_off;       // index of its per-channel scales in the scale array (-1: none)
};

struct Shape { int c, h, w; bool flat; int n; };

struct Parsed {
    std::vector<TensorSpec> tensors;
    std::vector<Shape> shapes;   // after each layer
    int64_t weights_bytes = 0, n_scales = 0, n_act_scales = 0;
    bool has_lstm = false;
    int feat = 0;
};

int parse_arch(const accerl_arch* a, Parsed& P) {
    if (!a) return fail(ACCERL_EINVAL, "arch is NULL");
    if (a->n_layers < 0 || a->n_layers > ACCERL_MAX_LAYERS) return fail(ACCERL_EINVAL, "n_layers out of range");
    if (a->n_actions < 1 || a->n_actions > 63) return fail(ACCERL_EINVAL, "n_actions must be 1..63");
    if (a->precision < ACCERL_INT8 || a->precision > ACCERL_BF16) return fail(ACCERL_EINVAL, "bad precision");
    if (a->obs_dtype != ACCERL_OBS_U8 && a->obs_dtype != ACCERL_OBS_F32) return fail(ACCERL_EINVAL, "bad obs_dtype");
    if (a->obs_c < 1 || a->obs_h < 1 || a->obs_w < 1) return fail(ACCERL_EINVAL, "bad observation shape");
    const bool q = a->precision == ACCERL_INT8;
    Shape s;
    if (a->obs_h == 1 && a->obs_w == 1) s = Shape{0, 0, 0, true, a->obs_c};
    else s = Shape{a->obs_c, a->obs_h, a->obs_w, false, 0};
    for (int i = 0; i < a->n_layers; ++i) if (a->layers[i].kind == ACCERL_LSTM) P.has_lstm = true;
    int64_t off = 0;
    int64_t n_act = 1, n_sw = 0;
    auto add = [&](int layer, int sub, int64_t rows, int64_t cols, bool bias, WType wt) {
        TensorSpec t{layer, sub, rows, cols, bias, wt, 0, -1, -1};
        off = up(off, 16);
        t.w_off = off;
        off += rows * cols * (wt == W_I8 ? 1 : 4);
        if (bias) { off = up(off, 16); t.b_off = off; off += rows * 4; }
        if (wt == W_I8) { t.sw_off = n_sw; n_sw += rows; }
        P.tensors.push_back(t);
    };
    for (int i = 0; i < a->n_layers; ++i) {
        const accerl_layer& L = a->layers[i];
        switch (L.kind) {
            case ACCERL_CONV:
                if (s.flat) return fail(ACCERL_EINVAL, "layer %d: conv on a flat tensor", i);
                if (L.cin != s.c || L.cout < 1 || L.k < 1 || L.stride < 1 || L.pad < 0 || L.pad >= L.k)
                    return fail(ACCERL_EINVAL, "layer %d: inconsistent conv", i);
                if (s.h + 2 * L.pad < L.k || s.w + 2 * L.pad < L.k) return fail(ACCERL_EINVAL, "layer %d: kernel larger than input", i);
                add(i, 0, L.cout, (int64_t)L.cin * L.k * L.k, true, q ? W_I8 : W_F32);
                s = Shape{L.cout, out_hw(s.h, L.k, L.stride, L.pad), out_hw(s.w, L.k, L.stride, L.pad), false, 0};
                n_act += 1;
                break;
            case ACCERL_DENSE:
                if (!s.flat || L.cin != s.n || L.cout < 1) return fail(ACCERL_EINVAL, "layer %d: inconsistent dense", i);
                add(i, 0, L.cout, L.cin, true, q ? W_I8 : W_F32);
                s = Shape{0, 0, 0, true, L.cout};
                n_act += 1;
                break;
            case ACCERL_MAXPOOL:
                if (s.flat || L.k < 1 || L.stride < 1 || L.pad < 0 || 2 * L.pad > L.k || s.h + 2 * L.pad < L.k || s.w + 2 * L.pad < L.k)
                    return fail(ACCERL_EINVAL, "layer %d: inconsistent maxpool", i);
                s = Shape{s.c, out_hw(s.h, L.k, L.stride, L.pad), out_hw(s.w, L.k, L.stride, L.pad), false, 0};
                break;
            case ACCERL_RESBLOCK:
                if (s.flat || L.cin != s.c || L.cout != s.c) return fail(ACCERL_EINVAL, "layer %d: inconsistent resblock", i);
                add(i, 0, s.c, (int64_t)s.c * 9, true, q ? W_I8 : W_F32);
                add(i, 1, s.c, (int64_t)s.c * 9, true, q ? W_I8 : W_F32);
                n_act += 2;
                break;
            case ACCERL_RELU:
                break;
            case ACCERL_FLATTEN:
                if (!s.flat) s = Shape{0, 0, 0, true, s.c * s.h * s.w};
                break;
            case ACCERL_LSTM:
                if (!s.flat || L.cin != s.n || L.cout < 1) return fail(ACCERL_EINVAL, "layer %d: inconsistent lstm", i);
                if (i != a->n_layers - 1) return fail(ACCERL_EUNSUPPORTED, "layer %d: the lstm must be the last layer", i);
                add(i, 0, 4 * (int64_t)L.cout, L.cin, true, W_F32);
                add(i, 1, 4 * (int64_t)L.cout, L.cout, false, W_F32);
                s = Shape{0, 0, 0, true, L.cout};
                break;
            default:
                return fail(ACCERL_EINVAL, "layer %d: unknown kind %d", i, L.kind);
        }
        P.shapes.push_back(s);
    }
    if (!s.flat) return fail(ACCERL_EINVAL, "the heads need a flat feature vector (add a flatten layer)");
    P.feat = s.n;
    add(a->n_layers, 0, a->n_actions + 1, s.n, true, (q && !P.has_lstm) ? W_I8 : W_F32);
    P.weights_bytes = off;
    P.n_act_scales = q ? n_act : 0;
    P.n_scales = q ? n_act + n_sw : 0;
    return ACCERL_OK;
}

// ------------------------------------------------------------------ plan
enum StepKind { ST_MLP, ST_QUANT_OBS, ST_CONV, ST_GEMM, ST_GEMM_F32, ST_MAXPOOL, ST_LSTM_PACK, ST_SAMPLE, ST_HEADS };

struct Step {
    StepKind kind;
    int layer = -1, sub = 0;
    int in_buf = -1, out_buf = -1, res_buf = -1;   // -1 = the caller's states (in) / none
    int pool_buf = -1;          // conv: output of the max-pool fused into it (-1 = none)
    bool fused = false;         // maxpool: normally done by the conv step before it
    bool fuse_next = false;     // conv: normally runs together with the conv step after it (its output stays on chip)
    bool fused_prev = false;    // conv: normally done by the conv step before it
    bool resblock = false;      // conv with fuse_next: the pair is a residual block (skip connection from this step's input)
    bool stack_head = false;    // conv: normally runs together with its max-pool and the two residual blocks behind it (steps +1 .. +5)
    bool stack_member = false;  // max-pool / conv: normally done by the stack kernel of an earlier step
    ConvParams cp{};
    Elem el = EL_I8;
    int NT = 1, KS = 0, RD = 16, PF = 16;
    GemmParams gp{};
    GemmEpi epi = EPI_REQUANT;
    GemmF32Params fp{};
    LstmPackParams lp{};
    MlpParams mp{};
    // maxpool
    int H = 0, W = 0, Cs = 0, Ho = 0, Wo = 0, k = 0, s = 0, pad = 0;
    float inv_s0 = 0.f;
    int D = 0, Dpad = 0;
    // offsets into the device constant block
    int64_t o_w = -1, o_bias = -1, o_mult = -1, o_lut = -1;
    // what the step's output is, for taps
    int64_t out_elems = 0;      // stored elements per state
    int64_t acc_elems = 0;      // int32 accumulator elements per state (0 = none)
};

struct Buf { int64_t per_state; int64_t off; int slot[2]; };   // slot in the normal / the debug layout

}  // namespace

struct accerl_policy {
    accerl_arch arch;
    Parsed P;
    int device = 0;
    std::vector<Step> steps;
    std::vector<Buf> bufs;
    // workspace slots (bytes per state); buffers whose lifetimes do not overlap share one.  Layout 0 serves
    // forward calls; layout 1 serves debug calls, which may run a conv and its max-pool as separate steps.
    std::vector<int64_t> slots[2];
    int ws_layout = 0;
    int64_t ws_per_state = 0;
    char* consts = nullptr;
    char* ws = nullptr;
    int64_t ws_states = 0;
    int64_t chunk = 0;
    int64_t obs_bytes = 0;
    bool recurrent = false;
    int lstm_hidden = 0;
    // policy mixture (owned by the smaller policy of a pair): compacted inputs and results of both subsets,
    // and a ring of pinned host buffers for the row lists
    char* mix_dev = nullptr;
    int64_t mix_rows = 0;
    int32_t* mix_pin[4] = {nullptr, nullptr, nullptr, nullptr};
    hipEvent_t mix_ev[4] = {nullptr, nullptr, nullptr, nullptr};
    int64_t mix_pin_rows = 0;
    int mix_slot = 0;
    // measurement aid while profiling is on: one event after every launch (and one before the first of a
    // pass); a step's time is the span between the event before it and the event after it
    bool profiling = false;
    struct Ev { int step; hipEvent_t a, b; };
    std::vector<Ev> events;
    std::vector<hipEvent_t> ev_starts;
};

namespace {

struct Builder {
    const accerl_arch* a;
    const Parsed& P;
    const char* wblob;
    const float* scales;
    accerl_policy* pol;
    std::vector<char> cst;      // host image of the device constant block

    int64_t put(const void* src, int64_t bytes) {
        const int64_t o = up((int64_t)cst.size(), 256);
        cst.resize(o + bytes);
        if (src) memcpy(cst.data() + o, src, bytes);
        else memset(cst.data() + o, 0, bytes);
        return o;
    }
    int new_buf(int64_t per_state) {
        pol->bufs.push_back(Buf{up(per_state, 16), 0, {-1, -1}});
        return (int)pol->bufs.size() - 1;
    }
    const TensorSpec& tensor(int layer, int sub) const {
        for (const auto& t : P.tensors) if (t.layer == layer && t.sub == sub) return t;
        return P.tensors.back();
    }
    const int8_t* wq(const TensorSpec& t) const { return (const int8_t*)(wblob + t.w_off); }
    const float* wf(const TensorSpec& t) const { return (const float*)(wblob + t.w_off); }
    const float* bias(const TensorSpec& t) const { return (const float*)(wblob + t.b_off); }
    const float* sw(const TensorSpec& t) const { return scales + P.n_act_scales + t.sw_off; }

    static int32_t biasq(float b, float s_in, float s_w) {
        return (int32_t)std::rint((double)b / ((double)s_in * (double)s_w));
    }
    static float mult(float s_in, float s_w, float s_out) {
        return (float)(((double)s_in * (double)s_w) / (double)s_out);
    }
};

uint32_t magic_of(int d) { return d <= 1 ? 0u : (uint32_t)((0x100000000ull + (uint64_t)d - 1) / (uint64_t)d); }
int gcd_int(int a, int b) { while (b) { const int t = a % b; a = b; b = t; } return a; }

// One convolution (a conv layer or half of a resblock) -> a conv step.
int plan_conv(Builder& B, int layer, int sub, const TensorSpec& t, Elem el, bool src_u8,
              int Cin, int H, int W, int Cout, int k, int s, int pad, bool relu, bool relu_in,
              int in_buf, int out_buf, int res_buf, float s_in, float s_out, float s_res, int pool_buf = -1) {
    Step st;
    st.kind = ST_CONV;
    st.layer = layer;
    st.sub = sub;
    st.in_buf = in_buf;
    st.out_buf = out_buf;
    st.res_buf = res_buf;
    st.el = el;
    const int esz = el == EL_I8 ? 1 : 2;
    bool pool = pool_buf >= 0;                       // fuse the 3x3 stride-2 pad-1 max-pool that follows
    const int Cs_out = (int)up(Cout, 4);
    if (src_u8 && Cin > 4) return fail(ACCERL_EUNSUPPORTED, "uint8 observations with more than 4 channels");
    if (src_u8 && (W & 3)) return fail(ACCERL_EUNSUPPORTED, "uint8 observation width must be a multiple of 4");
    const int Ho = out_hw(H, k, s, pad), Wo_img = out_hw(W, k, s, pad);
    // Thin layers (at most 8 stored output channels): P horizontally adjacent output pixels are computed
    // as one pixel of a layer with P times the channels, a kernel row wider by (P-1) strides (zero weights
    // where a tap lies outside a pixel's own window) and P times the horizontal stride.  The bytes written
    // are the same channels-last image; every MFMA row and every epilogue lane then does useful work.
    int P = 1;
    if (Cs_out <= 8 && !getenv("ACCERL_NO_PIXEL_PACK")) {
        P = 16 / Cs_out;
        while (P > 1 && (Wo_img % P)) P >>= 1;
    }
    const int Cs_img = Cs_out;                      // stored channels per real output pixel
    const int CoutK = P > 1 ? P * Cs_img : Cout;    // channels of the layer the kernel sees
    const int Cs_outK = P > 1 ? P * Cs_img : Cs_out;
    const int Wo = Wo_img / P;
    const int kw = k + (P - 1) * s, sx = P * s;
    const int NT = (CoutK <= 16) ? 1 : (CoutK <= 32) ? 2 : (CoutK <= 64) ? 4 : 0;
    if (!NT) return fail(ACCERL_EUNSUPPORTED, "layer %d: more than 64 output channels", layer);
    const int Cs_in = (int)up(Cin, 4);
    const int pix = Cs_in * esz;
    const int kk = k, ss = s;
    const int Wt = W, Ht = H;
    const int run = kw * pix;                       // bytes of one kernel row of one (packed) pixel
    const int cpr = (run + 15) / 16;
    const int chunks = kk * cpr;
    const int k_steps = (chunks + 3) / 4;
    const int w_bytes = k_steps * NT * 1024;
    const int row_bytes = Wt * pix;

    ConvParams& c = st.cp;
    int mode, pitch;
    if (src_u8) { mode = CM_U8T; pitch = (int)up((int64_t)(W + 2 * pad) * pix, 16); }
    else if (pad == 0 && ((H * row_bytes) % 16) == 0) { mode = CM_FLAT; pitch = row_bytes; }
    else { mode = (row_bytes % 16) == 0 ? CM_ROWSV : CM_ROWS; pitch = (int)up((int64_t)(W + 2 * pad) * pix, 16); }
    const bool whole = mode == CM_FLAT;             // tiles are whole images, staged contiguously
    const bool rows_vec = mode == CM_ROWSV;         // image rows are whole 16-byte units (else gathered by dwords)

    int RD = [&] { int al = gcd_int(16, gcd_int(sx * pix, pitch)); return al < 4 ? 4 : al; }();
    const int w_lds_max = w_bytes + k_steps * 16 + CONV_LDS_CONST;
    const int PT = conv_pixel_tiles(NT);

    // band height: units to stage per tile <= 4096 (16 per lane), LDS within budget
    const int lds_cap = 160 * 1024 - 2048;
    int budget = 64 * 1024;
    if (w_lds_max + 40 * 1024 > budget) budget = w_lds_max + 40 * 1024;
    if (budget > lds_cap) budget = lds_cap;
    auto rows_of = [&](int th) { return (th - 1) * ss + kk; };
    auto tile_of = [&](int th) { return whole ? Ht * row_bytes : (int)up((int64_t)rows_of(th) * pitch, 16); };
    auto units_of = [&](int th) {
        if (whole) return tile_of(th) / 16;
        if (mode == CM_U8T) return rows_of(th) * (W / 4);
        return rows_of(th) * (rows_vec ? row_bytes / 16 : pitch / 16);
    };
    // Thin layers (one channel tile, a few MFMA steps) are bound by the vector instructions around the
    // MFMAs: they get small batches, so that the kernel needs few staging registers and four workgroups
    // share a compute unit.
    const bool thin = NT == 1 && k_steps <= 3 && !getenv("ACCERL_NO_THIN");
    const int thin_units = 1024;
    const int band_units = thin ? thin_units : 4096;
    if (thin) {   // LDS per workgroup small enough for several workgroups per compute unit
        const int thin_lds = 32 * 1024;
        if (budget > thin_lds) budget = thin_lds;
    }
    // fused pooling: the requantized conv rows of a band wait in LDS for the pooling pass
    const int pool_pix = Cs_out * esz;               // bytes per stored output pixel
    const int pool_unit = (pool_pix % 16) == 0 ? 16 : 8;
    int pool_ush = 0;
    while ((pool_unit << pool_ush) < pool_pix) ++pool_ush;
    if (pool && ((pool_pix % 8) != 0 || (pool_unit << pool_ush) != pool_pix || res_buf >= 0)) pool = false;
    const int PH = pool ? out_hw(Ho, 3, 2, 1) : 0, PW = pool ? out_hw(Wo_img, 3, 2, 1) : 0;
    auto conv_rows = [&](int tph) { return 2 * tph + 1 < Ho ? 2 * tph + 1 : Ho; };
    auto otile_of = [&](int th) { return (pool ? th * Wo_img * pool_pix : 0) + 8 * th * Wo + 16; };   // + the pixel table
    int TH = Ho, TPH = PH;
    if (pool) {
        if (!whole)
            while (TPH > 1 && (units_of(conv_rows(TPH)) > band_units ||
                               w_lds_max + tile_of(conv_rows(TPH)) + otile_of(conv_rows(TPH)) + 32 > budget)) --TPH;
        const int nb = (PH + TPH - 1) / TPH;
        TPH = (PH + nb - 1) / nb;
        TH = conv_rows(TPH);
        if (units_of(TH) > 4096 || w_lds_max + tile_of(TH) + otile_of(TH) + 32 > lds_cap) { pool = false; TH = Ho; TPH = 0; }
    }
    if (!pool && !whole) {
        while (TH > 1 && (units_of(TH) > band_units || w_lds_max + tile_of(TH) + otile_of(TH) + 32 > budget)) --TH;
        const int nb = (Ho + TH - 1) / TH;
        TH = (Ho + nb - 1) / nb;
    }
    if (units_of(TH) > 4096 || w_lds_max + tile_of(TH) + otile_of(TH) + 32 > lds_cap)   // (a whole thin image may exceed its soft cap)
        return fail(ACCERL_EUNSUPPORTED, "layer %d: one input band does not fit the staging limits", layer);
    const int n_bands = pool ? (PH + TPH - 1) / TPH : (Ho + TH - 1) / TH;
    const int tile_stride = tile_of(TH), units_img = units_of(TH), n_pix = TH * Wo;
    // images per batch: best use of the pixel-tile slots (4 waves x PT tiles of 16) a workgroup fills per round
    int G = 1;
    if (n_bands == 1) {
        const int slot = 4 * PT * 16;
        const int unit_cap = thin ? thin_units : 2560;
        // largest batch whose tile-slot use is within 3 % of the best one: more pixels per barrier pair
        double best = -1.0;
        auto util_of = [&](int gg) { return (double)gg * n_pix / ((gg * n_pix + slot - 1) / slot * slot); };
        int gmax = 1;
        for (int gg = 2; gg <= 64; ++gg) {
            if (gg * units_img > unit_cap || w_lds_max + gg * (tile_stride + otile_of(TH)) + 32 > budget) break;
            gmax = gg;
        }
        for (int gg = 1; gg <= gmax; ++gg) best = util_of(gg) > best ? util_of(gg) : best;
        for (int gg = 1; gg <= gmax; ++gg) if (util_of(gg) >= best - 0.03) G = gg;
    }
    // wave-private kernel for plain-copy tiles with LDS weights: 8 wavefronts, each with its own images
    int wp_G = 0, wp_PT = 0, wp_wave_tiles = 0;
    if (el == EL_I8 && mode == CM_FLAT && NT == 4 && n_bands == 1 && !pool && res_buf < 0 && !getenv("ACCERL_NO_WAVE_PRIVATE")) {
        double best = -1.0;
        for (int gg = 1; gg <= 8; ++gg) {
            const int wt = (int)up((int64_t)gg * tile_stride + 32, 16);
            if (w_lds_max + CONV_WP_NWAVES * wt + 8 * gg * n_pix + 16 > lds_cap) break;
            for (int pt = 4; pt >= 3; --pt) {
                if (!conv_wp_available(el, NT, RD, pt, gg * units_img)) continue;
                const int tiles = (gg * n_pix + 15) / 16, slots = (tiles + pt - 1) / pt * pt;
                const double util = (double)gg * n_pix / (slots * 16.0);
                if (util > best + 1e-9) { best = util; wp_G = gg; wp_PT = pt; wp_wave_tiles = wt; }
            }
        }
    }
    int KS = 0, PF = 16;
    if (wp_G) { G = wp_G; }
    else if (!conv_pick_variant(el, NT, k_steps, RD, mode, (G * units_img + 255) / 256, res_buf >= 0 || pool, &KS, &PF))
        return fail(ACCERL_EUNSUPPORTED, "layer %d: no convolution kernel covers this shape", layer);
    if (!KS && RD == 8) RD = 4;                     // the generic LDS-weight kernels read chunks at 16 or 4 bytes
    c.H = H; c.W = W; c.Cin_real = Cin; c.Cs_in = Cs_in; c.Ho = Ho; c.Wo = Wo; c.Cs_out = Cs_outK;
    c.k = kk; c.s = ss; c.sx = sx; c.pad = pad; c.TH = TH; c.n_bands = n_bands;
    c.in_rows = whole ? Ht : rows_of(TH); c.pitch = pitch; c.tile_stride = tile_stride;
    c.lds_tiles = wp_G ? CONV_WP_NWAVES * wp_wave_tiles : G * tile_stride + 32;
    c.wave_private = wp_G ? 1 : 0; c.wave_tiles = wp_wave_tiles; c.wp_pt = wp_PT;
    c.cpr = cpr; c.k_steps = k_steps; c.w_bytes = w_bytes;
    c.relu_in = relu_in; c.relu = relu; c.src_u8 = src_u8;
    c.mode = mode; c.G = G;
    c.img_bytes = H * row_bytes;
    c.units_img = units_img;
    c.row_units = mode == CM_U8T ? W / 4 : rows_vec ? row_bytes / 16 : pitch / 16;
    if ((int64_t)G * n_pix >= (1 << 20) || (int64_t)Ho * Wo >= (1 << 20) || tile_stride >= (1 << 23) || (int64_t)ss * pitch >= (1 << 23))
        return fail(ACCERL_EUNSUPPORTED, "layer %d: image too large for the pixel index arithmetic", layer);
    c.pool = pool ? 1 : 0; c.pool_out = nullptr; c.PH = PH; c.PW = PW; c.TPH = TPH; c.pool_W = Wo_img;
    c.pool_unit = pool_unit; c.pool_ush = pool_ush; c.lds_otile = pool ? G * TH * Wo_img * pool_pix : 0;
    c.lds_tab = (int)up((int64_t)8 * G * n_pix, 16);
    if (pool) { const int rowu = PW << pool_ush; c.inv_prow = 1.0f / (float)rowu; c.hinv_prow = 0.5f / (float)rowu; }
    st.pool_buf = pool ? pool_buf : -1;
    c.inv_wo = 1.0f / (float)Wo; c.hinv_wo = 0.5f / (float)Wo;
    c.magic_units = magic_of(units_img); c.magic_rowunits = magic_of(c.row_units);
    st.NT = NT; st.KS = KS; st.RD = RD; st.PF = PF;
    st.out_elems = (int64_t)Ho * Wo * Cs_outK;
    st.acc_elems = el == EL_I8 ? st.out_elems : 0;

    // ---- weight fragments: [k_step][n_tile][lane][16 bytes]; MFMA row i of tile tt is channel
    //      4*NT*(i/4) + 4*tt + i%4, so that a lane's accumulators are consecutive channels
    std::vector<char> frag((size_t)w_bytes, 0);
    const int epc = 16 / esz;                       // elements per chunk
    std::vector<int64_t> wsum(NT * 16, 0), wpos(NT * 16, 0), wabs(NT * 16, 0);
    for (int stp = 0; stp < k_steps; ++stp)
        for (int tt = 0; tt < NT; ++tt)
            for (int lane = 0; lane < 64; ++lane) {
                const int i = lane & 15, g = lane >> 4;
                const int n = 4 * NT * (i >> 2) + 4 * tt + (i & 3);
                const int q = 4 * stp + g;
                if (n >= CoutK) continue;
                const int dx = n / Cs_img, ch = n - dx * Cs_img;   // packed pixel and its channel (dx = 0 unpacked)
                if (ch >= Cout) continue;
                char* dst = frag.data() + ((size_t)(stp * NT + tt) * 64 + lane) * 16;
                for (int e = 0; e < epc; ++e) {
                    int ci, ky, kx;
                    {
                        const int kby = q / cpr;
                        const int idx = (q - kby * cpr) * epc + e;  // element index inside the kernel row run
                        const int kbx = idx / Cs_in, rem = idx - kbx * Cs_in;
                        ky = kby; kx = kbx; ci = rem;
                    }
                    kx -= dx * s;                               // tap inside this pixel's own window
                    if (ky >= k || kx < 0 || kx >= k || ci >= Cin) continue;
                    const int64_t src = (((int64_t)ch * Cin + ci) * k + ky) * k + kx;
                    if (el == EL_I8) {
                        const int8_t v = B.wq(t)[src];
                        dst[e] = (char)v;
                        wsum[n] += v;
                        wpos[n] += v > 0 ? v : 0;
                        wabs[n] += v > 0 ? v : -v;
                    } else {
                        const uint16_t v = host_bf16(B.wf(t)[src]);
                        memcpy(dst + 2 * e, &v, 2);
                    }
                }
            }
    st.o_w = B.put(frag.data(), w_bytes);
    if (el == EL_I8) {
        std::vector<int32_t> bq(NT * 16, 0);
        std::vector<float> ml(NT * 16, 0.f);
        bool pos23 = relu;
        for (int n = 0; n < CoutK; ++n) {
            const int ch = n % Cs_img;
            if (ch >= Cout) continue;
            int64_t b = Builder::biasq(B.bias(t)[ch], s_in, B.sw(t)[ch]);
            // the largest accumulator any input can produce: observations are 0 .. 255, activations -127 .. 127
            const int64_t top = b + (src_u8 ? 255 * wpos[n] : 127 * wabs[n]);
            if (top >= (1 << 23) || b <= -(1 << 30)) pos23 = false;
            if (src_u8) b += 128 * wsum[n];          // observations are staged as obs - 128
            bq[n] = (int32_t)b;
            ml[n] = Builder::mult(s_in, B.sw(t)[ch], s_out);
        }
        st.o_bias = B.put(bq.data(), bq.size() * 4);
        st.o_mult = B.put(ml.data(), ml.size() * 4);
        c.r = res_buf >= 0 ? (float)((double)s_res / (double)s_out) : 0.f;
        c.pos23 = pos23 ? 1 : 0;
    } else {
        std::vector<float> bf(NT * 16, 0.f);
        for (int n = 0; n < CoutK; ++n) if (n % Cs_img < Cout) bf[n] = B.bias(t)[n % Cs_img];
        st.o_bias = B.put(bf.data(), bf.size() * 4);
        if (src_u8) {
            // the staged value of an observation byte: bf16(v / 255).  The kernel computes it as bf16(float(v) * (1 / 255))
            // when that gives the same 256 values (it does with IEEE single arithmetic); a table is the fallback.
            std::vector<uint16_t> lut(256);
            bool same = true;
            const volatile float k255 = 1.0f / 255.0f;
            for (int v = 0; v < 256; ++v) {
                lut[v] = host_bf16((float)v / 255.0f);
                const volatile float prod = (float)v * k255;
                same = same && host_bf16(prod) == lut[v];
            }
            if (!same || getenv("ACCERL_OBS_LUT")) st.o_lut = B.put(lut.data(), 512);
        }
    }
    B.pol->steps.push_back(st);
    return ACCERL_OK;
}

// Fragments of a dense weight matrix: [n_tile][k_step][lane][16 bytes].  perm maps a stored input
// position to the logical input index (-1 = padding); rowmap maps a stored output row to the logical
// row (-1 = padding); get(n, k) returns the logical weight.
template <typename Get>
std::vector<char> gemm_frags(Elem el, int n_tiles, int k_steps, const std::vector<int>& perm,
                             const std::vector<int>& rowmap, Get get) {
    const int esz = el == EL_I8 ? 1 : 2, epc = 16 / esz;
    std::vector<char> frag((size_t)n_tiles * k_steps * 1024, 0);
    for (int nt = 0; nt < n_tiles; ++nt)
        for (int st = 0; st < k_steps; ++st)
            for (int lane = 0; lane < 64; ++lane) {
                const int nrow = 16 * nt + (lane & 15), g = lane >> 4;
                if (nrow >= (int)rowmap.size() || rowmap[nrow] < 0) continue;
                char* dst = frag.data() + ((size_t)(nt * k_steps + st) * 64 + lane) * 16;
                for (int e = 0; e < epc; ++e) {
                    const int pos = st * 4 * epc + g * epc + e;
                    if (pos >= (int)perm.size() || perm[pos] < 0) continue;
                    const double v = get(rowmap[nrow], perm[pos]);
                    if (el == EL_I8) dst[e] = (char)(int8_t)v;
                    else { const uint16_t h = host_bf16((float)v); memcpy(dst + 2 * e, &h, 2); }
                }
            }
    return frag;
}

struct Cursor {            // the tensor the next layer reads
    Shape shape;
    int buf = -1;          // -1 = the caller's states
    Elem el = EL_I8;
    float scale = 1.f;     // int8 activations
    bool relu_pending = false;
    std::vector<int> perm; // flat tensors: stored position -> logical index
    int stored = 0;        // stored elements per state (flat tensors)
};

int build_plan(Builder& B) {
    const accerl_arch* a = B.a;
    const Parsed& P = B.P;
    accerl_policy* pol = B.pol;
    const bool q = a->precision == ACCERL_INT8;
    const bool image = !(a->obs_h == 1 && a->obs_w == 1);
    pol->recurrent = P.has_lstm;
    pol->obs_bytes = (int64_t)a->obs_c * a->obs_h * a->obs_w * (a->obs_dtype == ACCERL_OBS_U8 ? 1 : 4);
    const float* act = B.scales;
    int ai = 0;
    if (q) {
        for (int64_t i = 0; i < P.n_scales; ++i)
            if (!(B.scales[i] > 0.f) || !std::isfinite(B.scales[i])) return fail(ACCERL_EINVAL, "quant_scales[%lld] is not a positive finite number", (long long)i);
        if (a->obs_dtype == ACCERL_OBS_U8 && act[0] != (float)(1.0 / 255.0))
            return fail(ACCERL_EINVAL, "uint8 observations need s_0 = 1/255");
    }
    if (image && a->obs_dtype != ACCERL_OBS_U8) return fail(ACCERL_EUNSUPPORTED, "image observations must be uint8");
    if (!image && a->obs_dtype != ACCERL_OBS_F32) return fail(ACCERL_EUNSUPPORTED, "vector observations must be fp32");
    if (image && a->precision == ACCERL_FP32) return fail(ACCERL_EUNSUPPORTED, "image networks run as int8 or bf16");
    if (!image && a->precision == ACCERL_BF16) return fail(ACCERL_EUNSUPPORTED, "vector-observation teachers run in fp32");

    // ---------------- fused int8 MLP: every layer dense, at most 64 wide
    if (q && !image && !P.has_lstm) {
        bool ok = a->n_layers >= 1 && a->n_layers <= MLP_MAX_LAYERS && a->obs_c <= 64;
        for (int i = 0; i < a->n_layers; ++i) ok = ok && a->layers[i].kind == ACCERL_DENSE && a->layers[i].cout <= 64;
        if (ok) {
            Step st;
            st.kind = ST_MLP;
            st.layer = 0;
            MlpParams& m = st.mp;
            m.D = a->obs_c; m.A = a->n_actions; m.n_hidden = a->n_layers;
            m.inv_s0 = (float)(1.0 / (double)act[0]);
            const int nl = a->n_layers + 1;
            std::vector<char> frag((size_t)nl * 4 * 1024, 0);
            std::vector<int32_t> bq((size_t)nl * 64, 0);
            std::vector<float> ml((size_t)nl * 64, 0.f);
            float s_in = act[0];
            int Kprev = a->obs_c;
            m.k32 = a->obs_c <= 32 ? 1 : 0;
            bool p23 = !getenv("ACCERL_NO_P23");
            for (int l = 0; l < nl; ++l) {
                const TensorSpec& t = B.tensor(l < a->n_layers ? l : a->n_layers, 0);
                const int N = (int)t.rows, K = (int)t.cols;
                const float s_out = l < a->n_layers ? act[1 + l] : 0.f;
                for (int tt = 0; tt < 4; ++tt)
                    for (int lane = 0; lane < 64; ++lane) {
                        const int n = 16 * tt + (lane & 15), g = lane >> 4;
                        if (n >= N) continue;
                        char* dst = frag.data() + ((size_t)(l * 4 + tt) * 64 + lane) * 16;
                        for (int e = 0; e < 16; ++e) {
                            // layer 0 reads features in natural order; later layers read the accumulator
                            // layout of the layer before: slot 4*t' + r of lane group g is unit 16t' + 4g + r
                            // (observations of at most 32 features go through the K = 32 MFMA: 8 features per lane group)
                            int k = (l == 0) ? 16 * g + e : 16 * (e >> 2) + 4 * g + (e & 3);
                            if (l == 0 && m.k32) k = (e < 8) ? 8 * g + e : K;
                            if (k < K) dst[e] = (char)B.wq(t)[(int64_t)n * K + k];
                        }
                    }
                for (int n = 0; n < N; ++n) {
                    bq[l * 64 + n] = Builder::biasq(B.bias(t)[n], s_in, B.sw(t)[n]);
                    ml[l * 64 + n] = l < a->n_layers ? Builder::mult(s_in, B.sw(t)[n], s_out)
                                                      : (float)((double)s_in * (double)B.sw(t)[n]);
                    if (l < a->n_layers) {   // the largest accumulator any input (-127 .. 127 per feature) can produce
                        int64_t wabs = 0;
                        for (int k = 0; k < K; ++k) { const int v = B.wq(t)[(int64_t)n * K + k]; wabs += v < 0 ? -v : v; }
                        const int64_t b = bq[l * 64 + n];
                        if (!a->layers[l].relu || b + 127 * wabs >= (1 << 23) || b <= -(1 << 30)) p23 = false;
                    }
                }
                if (l < a->n_layers) { m.lo[l] = a->layers[l].relu ? 0 : -127; s_in = s_out; }
                (void)Kprev; Kprev = N;
            }
            st.o_w = B.put(frag.data(), frag.size());
            st.o_bias = B.put(bq.data(), bq.size() * 4);
            st.o_mult = B.put(ml.data(), ml.size() * 4);
            // three-instruction requantization (see requant_relu4_p23): c = -2^23 * m, exact
            m.p23 = p23 ? 1 : 0;
            std::vector<float> cf((size_t)a->n_layers * 64, 0.f);
            for (size_t i = 0; i < cf.size(); ++i) cf[i] = ml[i] * -8388608.0f;
            st.o_lut = B.put(cf.data(), cf.size() * 4);
            pol->steps.push_back(st);
            return ACCERL_OK;
        }
    }

    // ---------------- fp32 teacher on vector observations: chain of fp32 dense layers
    if (a->precision == ACCERL_FP32) {
        int cur = -1, K = a->obs_c;
        for (int i = 0; i <= a->n_layers; ++i) {
            const bool heads = i == a->n_layers;
            if (!heads && a->layers[i].kind != ACCERL_DENSE) return fail(ACCERL_EUNSUPPORTED, "fp32 teachers are dense-only");
            const TensorSpec& t = B.tensor(i, 0);
            Step st;
            st.kind = ST_GEMM_F32;
            st.layer = i;
            st.in_buf = cur;
            GemmF32Params& f = st.fp;
            f.K = K; f.N = (int)t.rows; f.ldx = K; f.relu = heads ? 0 : a->layers[i].relu; f.heads = heads; f.A = a->n_actions;
            st.o_w = B.put(B.wf(t), t.rows * t.cols * 4);
            st.o_bias = B.put(B.bias(t), t.rows * 4);
            if (!heads) {
                st.out_buf = B.new_buf(t.rows * 4);
                f.ldo = (int)t.rows;
                st.out_elems = t.rows;
                cur = st.out_buf;
                K = (int)t.rows;
            }
            pol->steps.push_back(st);
        }
        Step ss; ss.kind = ST_SAMPLE; ss.layer = a->n_layers;
        pol->steps.push_back(ss);
        return ACCERL_OK;
    }

    // ---------------- general path: int8 student or bf16 teacher, layer by layer
    const Elem el = q ? EL_I8 : EL_BF16;
    const int esz = q ? 1 : 2;
    Cursor cur;
    cur.shape = image ? Shape{a->obs_c, a->obs_h, a->obs_w, false, 0} : Shape{0, 0, 0, true, a->obs_c};
    cur.el = el;
    if (q) cur.scale = act[ai++];
    int pool_prealloc = -1;       // output buffer made for the max-pool layer while planning the conv before it
    bool pool_fused = false;
    for (int i = 0; i < a->n_layers; ++i) {
        const accerl_layer& L = a->layers[i];
        switch (L.kind) {
            case ACCERL_CONV: {
                const Shape o = P.shapes[i];
                const int ob = B.new_buf((int64_t)o.h * o.w * up(o.c, 4) * esz);
                const float s_out = q ? act[ai++] : 0.f;
                // a 3x3 stride-2 pad-1 max-pool right after the conv is fused into its epilogue when it fits
                pool_prealloc = -1;
                if (i + 1 < a->n_layers && a->layers[i + 1].kind == ACCERL_MAXPOOL && a->layers[i + 1].k == 3 &&
                    a->layers[i + 1].stride == 2 && a->layers[i + 1].pad == 1 && !getenv("ACCERL_NO_POOL_FUSE")) {
                    const Shape po = P.shapes[i + 1];
                    pool_prealloc = B.new_buf((int64_t)po.h * po.w * up(po.c, 4) * esz);
                }
                int rc = plan_conv(B, i, 0, B.tensor(i, 0), el, cur.buf < 0, cur.shape.c, cur.shape.h, cur.shape.w,
                                   L.cout, L.k, L.stride, L.pad, L.relu != 0, cur.relu_pending, cur.buf, ob, -1,
                                   cur.scale, s_out, 0.f, pool_prealloc);
                if (rc) return rc;
                pool_fused = pol->steps.back().pool_buf >= 0;
                cur.shape = o; cur.buf = ob; cur.scale = s_out; cur.relu_pending = false;
                break;
            }
            case ACCERL_MAXPOOL: {
                if (cur.buf < 0) return fail(ACCERL_EUNSUPPORTED, "layer %d: pooling directly on the observation", i);
                if (cur.relu_pending) return fail(ACCERL_EUNSUPPORTED, "layer %d: relu directly before maxpool", i);
                const Shape o = P.shapes[i];
                Step st;
                st.kind = ST_MAXPOOL; st.layer = i; st.el = el;
                st.in_buf = cur.buf;
                st.H = cur.shape.h; st.W = cur.shape.w; st.Cs = (int)up(cur.shape.c, 4); st.Ho = o.h; st.Wo = o.w;
                st.k = L.k; st.s = L.stride; st.pad = L.pad;
                st.out_buf = pool_prealloc >= 0 ? pool_prealloc : B.new_buf((int64_t)o.h * o.w * st.Cs * esz);
                st.fused = pool_prealloc >= 0 && pool_fused;
                pool_prealloc = -1; pool_fused = false;
                st.out_elems = (int64_t)o.h * o.w * st.Cs;
                pol->steps.push_back(st);
                cur.shape = o; cur.buf = st.out_buf;
                break;
            }
            case ACCERL_RESBLOCK: {
                if (cur.buf < 0 || cur.relu_pending) return fail(ACCERL_EUNSUPPORTED, "layer %d: resblock needs a stored, un-rectified stream", i);
                const Shape sh = cur.shape;
                const int64_t bytes = (int64_t)sh.h * sh.w * up(sh.c, 4) * esz;
                const int mid = B.new_buf(bytes), ob = B.new_buf(bytes);
                const float s1 = q ? act[ai++] : 0.f, s_out = q ? act[ai++] : 0.f;
                int rc = plan_conv(B, i, 0, B.tensor(i, 0), el, false, sh.c, sh.h, sh.w, sh.c, 3, 1, 1, true, true,
                                   cur.buf, mid, -1, cur.scale, s1, 0.f);
                if (rc) return rc;
                rc = plan_conv(B, i, 1, B.tensor(i, 1), el, false, sh.c, sh.h, sh.w, sh.c, 3, 1, 1, false, false,
                               mid, ob, cur.buf, s1, s_out, cur.scale);
                if (rc) return rc;
                cur.buf = ob; cur.scale = s_out;
                break;
            }
            case ACCERL_RELU:
                cur.relu_pending = true;
                break;
            case ACCERL_FLATTEN: {
                if (cur.shape.flat) break;
                if (cur.buf < 0) return fail(ACCERL_EUNSUPPORTED, "flatten directly on the observation");
                const Shape sh = cur.shape;
                const int Cs = (int)up(sh.c, 4);
                cur.stored = sh.h * sh.w * Cs;
                cur.perm.assign(cur.stored, -1);
                for (int y = 0; y < sh.h; ++y)
                    for (int x = 0; x < sh.w; ++x)
                        for (int c = 0; c < sh.c; ++c) cur.perm[(y * sh.w + x) * Cs + c] = (c * sh.h + y) * sh.w + x;
                cur.shape = P.shapes[i];
                break;
            }
            case ACCERL_DENSE: {
                if (cur.buf < 0) {   // vector observation on the general path: quantize to padded int8 rows
                    if (!q) return fail(ACCERL_EUNSUPPORTED, "bf16 teacher on vector observations");
                    Step st;
                    st.kind = ST_QUANT_OBS; st.layer = -1;
                    st.D = a->obs_c; st.Dpad = (int)up(a->obs_c, 16);
                    st.inv_s0 = (float)(1.0 / (double)cur.scale);
                    st.out_buf = B.new_buf(st.Dpad);
                    st.out_elems = st.Dpad;
                    pol->steps.push_back(st);
                    cur.buf = st.out_buf; cur.stored = st.Dpad;
                    cur.perm.assign(st.Dpad, -1);
                    for (int k = 0; k < a->obs_c; ++k) cur.perm[k] = k;
                }
                const TensorSpec& t = B.tensor(i, 0);
                const int N = L.cout, Np = (int)up(N, 16 / esz), n_tiles = (N + 15) / 16;
                const int epm = 64 / esz, k_steps = (cur.stored + epm - 1) / epm;
                std::vector<int> rowmap(n_tiles * 16, -1);
                for (int n = 0; n < N; ++n) rowmap[n] = n;
                const int K = (int)t.cols;
                Step st;
                st.kind = ST_GEMM; st.layer = i; st.el = el;
                st.in_buf = cur.buf;
                st.out_buf = B.new_buf((int64_t)Np * esz);
                GemmParams& gp = st.gp;
                gp.Kp_bytes = cur.stored * esz; gp.k_steps = k_steps; gp.N = N; gp.Np = Np; gp.n_tiles = n_tiles;
                gp.relu_in = cur.relu_pending; gp.relu = L.relu;
                st.out_elems = Np;
                if (q) {
                    st.epi = EPI_REQUANT;
                    st.acc_elems = N;
                    const float s_out = act[ai++];
                    auto frag = gemm_frags(el, n_tiles, k_steps, cur.perm, rowmap, [&](int n, int k) { return (double)B.wq(t)[(int64_t)n * K + k]; });
                    st.o_w = B.put(frag.data(), frag.size());
                    std::vector<int32_t> bq(n_tiles * 16, 0);
                    std::vector<float> ml(n_tiles * 16, 0.f);
                    for (int n = 0; n < N; ++n) {
                        bq[n] = Builder::biasq(B.bias(t)[n], cur.scale, B.sw(t)[n]);
                        ml[n] = Builder::mult(cur.scale, B.sw(t)[n], s_out);
                    }
                    st.o_bias = B.put(bq.data(), bq.size() * 4);
                    st.o_mult = B.put(ml.data(), ml.size() * 4);
                    cur.scale = s_out;
                } else {
                    st.epi = EPI_BF16;
                    auto frag = gemm_frags(el, n_tiles, k_steps, cur.perm, rowmap, [&](int n, int k) { return (double)B.wf(t)[(int64_t)n * K + k]; });
                    st.o_w = B.put(frag.data(), frag.size());
                    std::vector<float> bf(n_tiles * 16, 0.f);
                    for (int n = 0; n < N; ++n) bf[n] = B.bias(t)[n];
                    st.o_bias = B.put(bf.data(), bf.size() * 4);
                }
                pol->steps.push_back(st);
                cur.buf = st.out_buf; cur.shape = P.shapes[i]; cur.relu_pending = false;
                cur.stored = Np;
                cur.perm.assign(Np, -1);
                for (int n = 0; n < N; ++n) cur.perm[n] = n;
                break;
            }
            case ACCERL_LSTM: {
                if (cur.buf < 0) return fail(ACCERL_EUNSUPPORTED, "lstm directly on the observation");
                const int In = L.cin, Hd = L.cout;
                if (Hd % 4) return fail(ACCERL_EUNSUPPORTED, "lstm hidden size must be a multiple of 4");
                for (int k = 0; k < In; ++k) if (cur.perm[k] != k) return fail(ACCERL_EUNSUPPORTED, "lstm input must be a plain vector");
                pol->lstm_hidden = Hd;
                const int Kx = In + Hd;
                Step pk;
                pk.kind = ST_LSTM_PACK; pk.layer = i; pk.sub = 0;
                pk.in_buf = cur.buf;
                pk.out_buf = B.new_buf((int64_t)Kx * 2);
                LstmPackParams& lp = pk.lp;
                lp.x_elem = cur.el; lp.x_scale = cur.scale; lp.x_pitch_bytes = cur.stored * esz; lp.x_relu = cur.relu_pending;
                lp.In = In; lp.Hd = Hd;
                pk.out_elems = Kx;
                pol->steps.push_back(pk);
                const TensorSpec& tih = B.tensor(i, 0);
                const TensorSpec& thh = B.tensor(i, 1);
                const int N = 4 * Hd, n_tiles = N / 16, k_steps = (Kx + 31) / 32;
                std::vector<int> perm(Kx), rowmap(N);
                for (int k = 0; k < Kx; ++k) perm[k] = k;
                for (int u = 0; u < Hd; ++u) for (int gt = 0; gt < 4; ++gt) rowmap[4 * u + gt] = gt * Hd + u;
                auto frag = gemm_frags(EL_BF16, n_tiles, k_steps, perm, rowmap, [&](int n, int k) {
                    return (double)(k < In ? B.wf(tih)[(int64_t)n * In + k] : B.wf(thh)[(int64_t)n * Hd + (k - In)]);
                });
                Step st;
                st.kind = ST_GEMM; st.layer = i; st.sub = 1; st.el = EL_BF16; st.epi = EPI_LSTM;
                st.in_buf = pk.out_buf;
                st.out_buf = B.new_buf((int64_t)Hd * 2);
                st.o_w = B.put(frag.data(), frag.size());
                std::vector<float> bf(N);
                for (int n = 0; n < N; ++n) bf[n] = B.bias(tih)[rowmap[n]];
                st.o_bias = B.put(bf.data(), bf.size() * 4);
                GemmParams& gp = st.gp;
                gp.Kp_bytes = Kx * 2; gp.k_steps = k_steps; gp.N = N; gp.Np = Hd; gp.n_tiles = n_tiles; gp.Hd = Hd;
                st.out_elems = Hd;
                pol->steps.push_back(st);
                cur.buf = st.out_buf; cur.el = EL_BF16; cur.shape = P.shapes[i]; cur.relu_pending = false;
                cur.stored = Hd;
                cur.perm.resize(Hd);
                for (int k = 0; k < Hd; ++k) cur.perm[k] = k;
                break;
            }
        }
    }
    // ---------------- heads + sampler
    {
        if (cur.buf < 0) return fail(ACCERL_EUNSUPPORTED, "a network needs at least one layer before the heads");
        const TensorSpec& t = B.tensor(a->n_layers, 0);
        const int A = a->n_actions, N = A + 1, n_tiles = (N + 15) / 16, K = (int)t.cols;
        const Elem hel = cur.el;
        const int hesz = hel == EL_I8 ? 1 : 2, epm = 64 / hesz, k_steps = (cur.stored + epm - 1) / epm;
        std::vector<int> rowmap(n_tiles * 16, -1);
        for (int n = 0; n < N; ++n) rowmap[n] = n;
        Step st;
        st.kind = ST_GEMM; st.layer = a->n_layers; st.el = hel;
        st.in_buf = cur.buf;
        GemmParams& gp = st.gp;
        gp.Kp_bytes = cur.stored * hesz; gp.k_steps = k_steps; gp.N = N; gp.Np = N; gp.n_tiles = n_tiles; gp.A = A;
        gp.relu_in = cur.relu_pending;
        if (hel == EL_I8) {
            st.epi = EPI_HEADS_I8;
            st.acc_elems = N;
            auto frag = gemm_frags(hel, n_tiles, k_steps, cur.perm, rowmap, [&](int n, int k) { return (double)B.wq(t)[(int64_t)n * K + k]; });
            st.o_w = B.put(frag.data(), frag.size());
            std::vector<int32_t> bq(n_tiles * 16, 0);
            std::vector<float> ml(n_tiles * 16, 0.f);
            for (int n = 0; n < N; ++n) {
                bq[n] = Builder::biasq(B.bias(t)[n], cur.scale, B.sw(t)[n]);
                ml[n] = (float)((double)cur.scale * (double)B.sw(t)[n]);
            }
            st.o_bias = B.put(bq.data(), bq.size() * 4);
            st.o_mult = B.put(ml.data(), ml.size() * 4);
        } else {
            st.epi = EPI_HEADS_F32ACC;
            auto frag = gemm_frags(hel, n_tiles, k_steps, cur.perm, rowmap, [&](int n, int k) { return (double)B.wf(t)[(int64_t)n * K + k]; });
            st.o_w = B.put(frag.data(), frag.size());
            std::vector<float> bf(n_tiles * 16, 0.f);
            for (int n = 0; n < N; ++n) bf[n] = B.bias(t)[n];
            st.o_bias = B.put(bf.data(), bf.size() * 4);
        }
        if (heads_supported(k_steps, gp.Kp_bytes, A)) {
            st.kind = ST_HEADS;                     // one kernel: heads GEMM + sampler
            pol->steps.push_back(st);
        } else {
            pol->steps.push_back(st);
            Step ss; ss.kind = ST_SAMPLE; ss.layer = a->n_layers;
            pol->steps.push_back(ss);
        }
    }
    return ACCERL_OK;
}

int ensure_workspace(accerl_policy* p, int64_t n, int layout, hipStream_t stream) {
    if (p->bufs.empty() || (n <= p->ws_states && layout == p->ws_layout)) return ACCERL_OK;
    if (n < p->ws_states) n = p->ws_states;
    if (p->ws) {
        HIP_TRY(hipStreamSynchronize(stream));
        HIP_TRY(hipDeviceSynchronize());
        HIP_TRY(hipFree(p->ws));
        p->ws = nullptr;
        p->ws_states = 0;
    }
    int64_t off = 0;
    const std::vector<int64_t>& sl = p->slots[layout];
    std::vector<int64_t> slot_off(sl.size());
    // (a buffer handed over in the fragment order of a dense layer holds whole tiles of 16 states)
    for (size_t i = 0; i < sl.size(); ++i) { slot_off[i] = off; off += up(sl[i] * up(n, 16) + 256, 256); }
    for (auto& b : p->bufs) b.off = b.slot[layout] >= 0 ? slot_off[b.slot[layout]] : -1;
    hipError_t e = hipMalloc((void**)&p->ws, (size_t)off);
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(ACCERL_ENOMEM, "workspace of %lld bytes: %s", (long long)off, hipGetErrorString(e)); }
    HIP_TRY(hipMemset(p->ws, 0, (size_t)off));
    p->ws_states = n;
    p->ws_layout = layout;
    return ACCERL_OK;
}

struct Call {
    const void* states; int64_t B; const float* uniforms; const uint8_t* done; float* h; float* c;
    float* logits; float* value; int32_t* action; hipStream_t stream;
    // debug
    bool debug = false; int layer = 0, tap = 0; void* out = nullptr; int64_t out_bytes = 0;
};

int find_tap_step(const accerl_policy* p, int layer, int tap, bool& is_acc) {
    const bool resblock = layer >= 0 && layer < p->arch.n_layers && p->arch.layers[layer].kind == ACCERL_RESBLOCK;
    is_acc = (tap == ACCERL_TAP_ACC || tap == ACCERL_TAP_ACC_A);
    if ((tap == ACCERL_TAP_ACC_A || tap == ACCERL_TAP_ACT_A) && !resblock) return -1;
    const int want_sub = resblock ? ((tap == ACCERL_TAP_ACC_A || tap == ACCERL_TAP_ACT_A) ? 0 : 1) : -1;
    int found = -1;
    for (int i = 0; i < (int)p->steps.size(); ++i) {
        const Step& s = p->steps[i];
        if (s.kind == ST_SAMPLE || s.layer != layer) continue;
        if (!is_acc && s.kind == ST_HEADS) continue;
        if (want_sub >= 0 && s.sub != want_sub) continue;
        if (is_acc && s.acc_elems == 0) continue;
        if (!is_acc && s.out_buf < 0) continue;
        found = i;
    }
    return found;
}

int run(accerl_policy* p, const Call& c) {
    if (c.B == 0) return ACCERL_OK;
    const accerl_arch& a = p->arch;
    const int A = a.n_actions;
    int last_step = (int)p->steps.size() - 1;
    bool tap_acc = false;
    int64_t tap_elems = 0, tap_esz = 0;
    const bool fused = p->steps.size() == 1 && p->steps[0].kind == ST_MLP;
    if (c.debug) {
        if (fused) {
            const int nl = a.n_layers;
            tap_acc = c.tap == ACCERL_TAP_ACC;
            if (c.tap != ACCERL_TAP_ACC && c.tap != ACCERL_TAP_ACT) return fail(ACCERL_EINVAL, "tap kind not available for this layer");
            if (c.layer < -1 || c.layer > nl || (c.layer == -1 && tap_acc) || (c.layer == nl && !tap_acc))
                return fail(ACCERL_EINVAL, "no such tap");
            tap_elems = c.layer == -1 ? a.obs_c : c.layer == nl ? A + 1 : a.layers[c.layer].cout;
            tap_esz = tap_acc ? 4 : 1;
        } else {
            last_step = find_tap_step(p, c.layer, c.tap, tap_acc);
            if (last_step < 0) return fail(ACCERL_EINVAL, "layer %d has no such tap", c.layer);
            const Step& s = p->steps[last_step];
            tap_elems = tap_acc ? s.acc_elems : s.out_elems;
            if (!tap_acc && s.kind == ST_GEMM) {
                // int8 rows are copied out without their padding; bf16 rows are converted whole, so they must have none
                if (s.epi != EPI_REQUANT && !(s.epi == EPI_BF16 && s.gp.N == s.gp.Np))
                    return fail(ACCERL_EINVAL, "layer %d: activation tap not available", c.layer);
                tap_elems = s.gp.N;
            }
            tap_esz = tap_acc ? 4 : (a.precision == ACCERL_INT8 && s.el == EL_I8 && s.kind != ST_LSTM_PACK) ? 1 : 4;
        }
        if (c.out_bytes != c.B * tap_elems * tap_esz)
            return fail(ACCERL_EINVAL, "tap needs %lld bytes, got %lld", (long long)(c.B * tap_elems * tap_esz), (long long)c.out_bytes);
    }
    int64_t chunk = p->chunk > 0 ? p->chunk : c.B;
    if (chunk > c.B) chunk = c.B;
    int rc = ensure_workspace(p, chunk, c.debug ? 1 : 0, c.stream);
    if (rc) return rc;
    for (int64_t c0 = 0; c0 < c.B; c0 += chunk) {
        const int64_t n = (c.B - c0 < chunk) ? (c.B - c0) : chunk;
        const char* states = (const char*)c.states + c0 * p->obs_bytes;
        float* logits = c.logits ? c.logits + c0 * A : nullptr;
        float* value = c.value ? c.value + c0 : nullptr;
        int32_t* action = c.action ? c.action + c0 : nullptr;
        const float* uni = c.uniforms ? c.uniforms + c0 : nullptr;
        char* tap_out = c.debug ? (char*)c.out + c0 * tap_elems * tap_esz : nullptr;
        auto bufp = [&](int b) -> char* { return b < 0 ? const_cast<char*>(states) : p->ws + p->bufs[b].off; };
        bool pooled = false;   // the last conv step also did the max-pool that follows it
        bool conv_pair_done = false;   // the last conv step also did the conv that follows it
        int stack_skip = 0;            // conv steps still to pass over: a stack kernel has done them
        hipEvent_t prof_prev = nullptr;
        for (int si = 0; si <= last_step; ++si) {
            const Step& s = p->steps[si];
            const bool tap_here = c.debug && !fused && si == last_step;
            hipError_t e = hipSuccess;
            bool launched = true;          // false for a step whose work the step before it has done
            if (p->profiling && !prof_prev) {
                HIP_TRY(hipEventCreate(&prof_prev));
                HIP_TRY(hipEventRecord(prof_prev, c.stream));
                p->ev_starts.push_back(prof_prev);
            }
            switch (s.kind) {
                case ST_MLP: {
                    MlpParams m = s.mp;
                    m.obs = (const float*)states; m.uniforms = uni; m.logits = logits; m.value = value; m.action = action;
                    m.B = n;
                    m.wfrag = (const v4i*)(p->consts + s.o_w);
                    m.bias = (const int32_t*)(p->consts + s.o_bias);
                    m.mult = (const float*)(p->consts + s.o_mult);
                    m.cfma = (const float*)(p->consts + s.o_lut);
                    m.tap_layer = -2; m.tap_acc = nullptr; m.tap_act = nullptr; m.tap_n = 0;
                    if (c.debug) {
                        m.tap_layer = c.layer; m.tap_n = (int)tap_elems;
                        if (tap_acc) m.tap_acc = (int32_t*)tap_out; else m.tap_act = (int8_t*)tap_out;
                    }
                    e = launch_mlp_i8(m, c.stream);
                    break;
                }
                case ST_QUANT_OBS:
                    e = launch_quant_obs((const float*)states, n, s.D, s.Dpad, s.inv_s0, (int8_t*)bufp(s.out_buf), c.stream);
                    break;
                case ST_CONV: {
                    if (stack_skip > 0) { --stack_skip; launched = false; break; }                             // done by the stack kernel
                    if (s.stack_head && !c.debug) {
                        ConvParams cv[5];
                        const int idx[5] = {si, si + 2, si + 3, si + 4, si + 5};
                        for (int k = 0; k < 5; ++k) {
                            const Step& t = p->steps[idx[k]];
                            cv[k] = t.cp;
                            cv[k].in = nullptr; cv[k].out = nullptr; cv[k].res = nullptr; cv[k].tap_acc = nullptr;
                            cv[k].wfrag = p->consts + t.o_w; cv[k].bias = p->consts + t.o_bias; cv[k].mult = (const float*)(p->consts + t.o_mult);
                            cv[k].B = n;
                        }
                        cv[0].in = bufp(s.in_buf);
                        cv[4].out = bufp(p->steps[si + 5].out_buf);
                        e = launch_stack(cv[0], cv[1], cv[2], cv[3], cv[4], c.stream);
                        pooled = true;          // the max-pool step behind this one is done too
                        stack_skip = 4;         // and so are the four convolutions of the two blocks
                        break;
                    }
                    if (s.fused_prev && conv_pair_done) { conv_pair_done = false; launched = false; break; }   // done by the step before
                    if (s.fuse_next && !c.debug) {
                        const Step& nx = p->steps[si + 1];
                        ConvParams ca = s.cp, cb = nx.cp;
                        ca.in = bufp(s.in_buf); ca.out = nullptr; ca.res = nullptr; ca.tap_acc = nullptr;
                        ca.wfrag = p->consts + s.o_w; ca.bias = p->consts + s.o_bias; ca.mult = (const float*)(p->consts + s.o_mult);
                        ca.B = n;
                        cb.in = nullptr; cb.out = bufp(nx.out_buf); cb.res = nullptr; cb.tap_acc = nullptr;
                        cb.wfrag = p->consts + nx.o_w; cb.bias = p->consts + nx.o_bias; cb.mult = (const float*)(p->consts + nx.o_mult);
                        cb.B = n;
                        e = s.resblock ? launch_resblock(ca, cb, c.stream) : launch_conv_fused(ca, s.NT, cb, c.stream);
                        conv_pair_done = true;
                        break;
                    }
                    ConvParams cp = s.cp;
                    cp.in = bufp(s.in_buf); cp.out = bufp(s.out_buf);
                    cp.res = s.res_buf >= 0 ? bufp(s.res_buf) : nullptr;
                    cp.tap_acc = (tap_here && tap_acc) ? (int32_t*)tap_out : nullptr;
                    cp.wfrag = p->consts + s.o_w;
                    cp.bias = p->consts + s.o_bias;
                    cp.mult = s.o_mult >= 0 ? (const float*)(p->consts + s.o_mult) : nullptr;
                    cp.lut = s.o_lut >= 0 ? (const uint16_t*)(p->consts + s.o_lut) : nullptr;
                    cp.B = n;
                    if (c.debug) cp.out_frag = 0;
                    // the fused max-pool is left out when this conv's own output is the tap
                    if (cp.pool && !tap_here) { cp.pool_out = bufp(s.pool_buf); pooled = true; }
                    else cp.pool = 0;
                    e = launch_conv(cp, s.el, s.NT, s.KS, s.RD, s.PF, c.stream);
                    break;
                }
                case ST_MAXPOOL:
                    if (s.fused && pooled) { pooled = false; launched = false; break; }   // done by the conv step before
                    e = launch_maxpool(bufp(s.in_buf), bufp(s.out_buf), n, s.H, s.W, s.Cs, s.Ho, s.Wo, s.k, s.s, s.pad, s.el, c.stream);
                    break;
                case ST_GEMM: {
                    GemmParams gp = s.gp;
                    gp.x = bufp(s.in_buf);
                    gp.out = s.out_buf >= 0 ? bufp(s.out_buf) : nullptr;
                    gp.wfrag = p->consts + s.o_w;
                    gp.bias = p->consts + s.o_bias;
                    gp.mult = s.o_mult >= 0 ? (const float*)(p->consts + s.o_mult) : nullptr;
                    gp.tap_acc = (tap_here && tap_acc) ? (int32_t*)tap_out : nullptr;
                    gp.logits = logits; gp.value = value;
                    gp.h = c.h ? c.h + c0 * p->lstm_hidden : nullptr;
                    gp.c = c.c ? c.c + c0 * p->lstm_hidden : nullptr;
                    gp.B = n;
                    if (c.debug) gp.x_frag = 0;
                    e = launch_gemm(gp, s.el, s.epi, c.stream);
                    break;
                }
                case ST_GEMM_F32: {
                    GemmF32Params f = s.fp;
                    f.x = (const float*)bufp(s.in_buf);
                    f.w = (const float*)(p->consts + s.o_w);
                    f.bias = (const float*)(p->consts + s.o_bias);
                    f.out = s.out_buf >= 0 ? (float*)bufp(s.out_buf) : nullptr;
                    f.logits = logits; f.value = value; f.B = n;
                    e = launch_gemm_f32(f, c.stream);
                    break;
                }
                case ST_LSTM_PACK: {
                    LstmPackParams lp = s.lp;
                    lp.x = bufp(s.in_buf);
                    lp.done = c.done ? c.done + c0 : nullptr;
                    lp.h = c.h + c0 * p->lstm_hidden; lp.c = c.c + c0 * p->lstm_hidden;
                    lp.xh = (uint16_t*)bufp(s.out_buf);
                    lp.B = n;
                    e = launch_lstm_pack(lp, c.stream);
                    break;
                }
                case ST_SAMPLE:
                    e = launch_sample(logits, uni, action, n, A, c.stream);
                    break;
                case ST_HEADS: {
                    HeadsParams hp{};
                    hp.x = bufp(s.in_buf);
                    hp.wfrag = p->consts + s.o_w;
                    hp.bias = p->consts + s.o_bias;
                    hp.mult = s.o_mult >= 0 ? (const float*)(p->consts + s.o_mult) : nullptr;
                    hp.uniforms = uni; hp.logits = logits; hp.value = value; hp.action = action;
                    hp.tap_acc = (tap_here && tap_acc) ? (int32_t*)tap_out : nullptr;
                    hp.B = n; hp.Kp_bytes = s.gp.Kp_bytes; hp.k_steps = s.gp.k_steps; hp.A = A; hp.relu_in = s.gp.relu_in;
                    e = launch_heads(hp, s.el, c.stream);
                    break;
                }
            }
            if (e != hipSuccess) return fail(ACCERL_EHIP, "step %d (kind %d, layer %d): %s", si, (int)s.kind, s.layer, hipGetErrorString(e));
            if (p->profiling && launched) {
                accerl_policy::Ev ev{si, prof_prev, nullptr};
                HIP_TRY(hipEventCreate(&ev.b));
                HIP_TRY(hipEventRecord(ev.b, c.stream));
                p->events.push_back(ev);
                prof_prev = ev.b;
            }
            if (tap_here && !tap_acc) {
                const char* src = bufp(s.out_buf);
                if (s.kind == ST_GEMM && s.epi == EPI_REQUANT) {
                    HIP_TRY(hipMemcpy2DAsync(tap_out, (size_t)s.gp.N, src, (size_t)s.gp.Np, (size_t)s.gp.N, (size_t)n,
                                             hipMemcpyDeviceToDevice, c.stream));
                } else if (tap_esz == 1 || s.kind == ST_GEMM_F32) {
                    HIP_TRY(hipMemcpyAsync(tap_out, src, (size_t)(n * tap_elems * tap_esz), hipMemcpyDeviceToDevice, c.stream));
                } else {
                    HIP_TRY(launch_bf16_to_f32((const uint16_t*)src, (float*)tap_out, n * tap_elems, c.stream));
                }
            }
        }
    }
    if (c.debug) HIP_TRY(hipStreamSynchronize(c.stream));
    return ACCERL_OK;
}

int check_common(accerl_policy* p, const void* states, int64_t B, bool need_outputs, const float* uniforms,
                 float* logits, float* value, int32_t* action) {
    if (!p) return fail(ACCERL_EINVAL, "policy is NULL");
    if (B < 0) return fail(ACCERL_EINVAL, "B is negative");
    if (B == 0) return ACCERL_OK;
    if (!states) return fail(ACCERL_EINVAL, "states is NULL");
    if ((uintptr_t)states & 15) return fail(ACCERL_EINVAL, "states is not 16-byte aligned");
    if (need_outputs) {
        if (!uniforms || !logits || !value || !action) return fail(ACCERL_EINVAL, "an output or uniforms pointer is NULL");
        if (((uintptr_t)uniforms | (uintptr_t)logits | (uintptr_t)value | (uintptr_t)action) & 15)
            return fail(ACCERL_EINVAL, "a device pointer is not 16-byte aligned");
    }
    return ACCERL_OK;
}

}  // namespace

extern "C" {

int accerl_blob_sizes(const accerl_arch* arch, int64_t* weights_bytes, int64_t* n_scales) {
    Parsed P;
    int rc = parse_arch(arch, P);
    if (rc) return rc;
    if (weights_bytes) *weights_bytes = P.weights_bytes;
    if (n_scales) *n_scales = P.n_scales;
    return ACCERL_OK;
}

// Host half of policy creation: parse, check, build the plan and the host image of the constants.
// Workspace slots.  A buffer lives from the step that writes it to the last step that reads it; two
// buffers share a slot only if one is dead before the step that first writes the other, so no kernel
// ever reads and writes the same memory.  Buffers are taken in order of first write and placed in the
// free slot that wastes least (a smaller free slot is grown before a new one is opened).
static void assign_slots(accerl_policy* pol, int layout) {
    const int nb = (int)pol->bufs.size(), ns = (int)pol->steps.size();
    std::vector<int> first(nb, ns), last(nb, -1);
    for (int si = 0; si < ns; ++si) {
        const Step& st = pol->steps[si];
        int touched[4] = {st.in_buf, st.res_buf, st.out_buf, -1};
        if (layout == 0 && st.kind == ST_CONV && st.pool_buf >= 0 && !st.stack_head) touched[2] = st.pool_buf;   // writes the pooled image only
        if (layout == 1 && st.kind == ST_CONV) touched[3] = st.pool_buf;                       // may run either way
        if (layout == 0 && st.stack_member) continue;                                           // done by the stack kernel
        if (layout == 0 && st.stack_head) touched[2] = pol->steps[si + 5].out_buf;              // reads its input, writes the stack's output
        if (layout == 0 && st.kind == ST_MAXPOOL && st.fused) continue;                         // never launched
        if (layout == 0 && st.kind == ST_CONV && st.fused_prev) continue;                       // done by the step before
        if (layout == 0 && st.kind == ST_CONV && st.fuse_next && !st.stack_head) touched[2] = pol->steps[si + 1].out_buf;
        for (int b : touched) {
            if (b < 0) continue;
            first[b] = std::min(first[b], si);
            last[b] = std::max(last[b], si);
        }
    }
    std::vector<int64_t>& slots = pol->slots[layout];
    slots.clear();
    std::vector<int> busy_until;
    std::vector<int> order(nb);
    for (int i = 0; i < nb; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return first[a] < first[b]; });
    for (int b : order) {
        pol->bufs[b].slot[layout] = -1;
        if (last[b] < 0) continue;                   // not used in this layout
        const int64_t need = pol->bufs[b].per_state;
        int pick = -1;
        for (int sl = 0; sl < (int)slots.size(); ++sl) {
            if (busy_until[sl] >= first[b]) continue;
            if (pick < 0) { pick = sl; continue; }
            const bool fits = slots[sl] >= need, pfits = slots[pick] >= need;
            if (fits && (!pfits || slots[sl] < slots[pick])) pick = sl;
            else if (!fits && !pfits && slots[sl] > slots[pick]) pick = sl;
        }
        if (pick < 0) { slots.push_back(0); busy_until.push_back(-1); pick = (int)slots.size() - 1; }
        slots[pick] = std::max(slots[pick], need);
        busy_until[pick] = last[b];
        pol->bufs[b].slot[layout] = pick;
    }
}

static int create_host(const accerl_arch* arch, const void* weights, int64_t weights_bytes,
                       const float* quant_scales, int64_t n_scales, accerl_policy* pol, std::vector<char>& cst) {
    if (!weights) return fail(ACCERL_EINVAL, "weights is NULL");
    int rc = parse_arch(arch, pol->P);
    if (rc) return rc;
    pol->arch = *arch;
    if (weights_bytes != pol->P.weights_bytes)
        return fail(ACCERL_EINVAL, "weight blob is %lld bytes, arch needs %lld", (long long)weights_bytes, (long long)pol->P.weights_bytes);
    if (n_scales != pol->P.n_scales || (n_scales > 0 && !quant_scales))
        return fail(ACCERL_EINVAL, "scale array has %lld entries, arch needs %lld", (long long)n_scales, (long long)pol->P.n_scales);
    if (arch->precision == ACCERL_INT8) {
        for (const auto& t : pol->P.tensors) {
            if (t.wt != W_I8) continue;
            const int8_t* w = (const int8_t*)((const char*)weights + t.w_off);
            for (int64_t i = 0; i < t.rows * t.cols; ++i)
                if (w[i] == -128) return fail(ACCERL_EINVAL, "int8 weight -128 is outside the symmetric range");
        }
    }
    Builder B{arch, pol->P, (const char*)weights, quant_scales, pol, {}};
    rc = build_plan(B);
    if (rc) return rc;
    cst.swap(B.cst);
    if (!getenv("ACCERL_NO_CONV_FUSE")) {
        for (size_t si = 0; si + 1 < pol->steps.size(); ++si) {
            Step& sa = pol->steps[si];
            Step& sb = pol->steps[si + 1];
            if (sa.kind != ST_CONV || sb.kind != ST_CONV || sa.el != EL_I8 || sb.el != EL_I8) continue;
            if (sa.fused_prev || sa.res_buf >= 0 || sb.res_buf >= 0 || sb.in_buf != sa.out_buf) continue;
            bool read_elsewhere = false;             // the first layer's output must have no other reader
            for (size_t sj = si + 2; sj < pol->steps.size(); ++sj)
                if (pol->steps[sj].in_buf == sa.out_buf || pol->steps[sj].res_buf == sa.out_buf) read_elsewhere = true;
            if (read_elsewhere) continue;
            if (conv_fused_supported(sa.cp, sa.NT, sa.KS, sa.RD, sb.cp, sb.NT, sb.KS, sb.RD)) { sa.fuse_next = true; sb.fused_prev = true; }
        }
    }
    // Residual blocks of the shapes the block kernel covers: both convolutions in one launch (the first one's output
    // has no other reader by construction: it is the block's inner tensor).
    if (!getenv("ACCERL_NO_RESBLOCK_FUSE")) {
        for (size_t si = 0; si + 1 < pol->steps.size(); ++si) {
            Step& sa = pol->steps[si];
            Step& sb = pol->steps[si + 1];
            if (sa.kind != ST_CONV || sb.kind != ST_CONV || sa.el != EL_I8 || sb.el != EL_I8) continue;
            if (sa.fused_prev || sa.fuse_next || sb.fuse_next || sa.res_buf >= 0 || sb.res_buf < 0) continue;
            if (sb.in_buf != sa.out_buf || sb.res_buf != sa.in_buf || sa.in_buf < 0 || sa.pool_buf >= 0 || sb.pool_buf >= 0) continue;
            bool read_elsewhere = false;
            for (size_t sj = si + 2; sj < pol->steps.size(); ++sj)
                if (pol->steps[sj].in_buf == sa.out_buf || pol->steps[sj].res_buf == sa.out_buf) read_elsewhere = true;
            if (read_elsewhere) continue;
            if (resblock_supported(sa.cp, sa.NT, sb.cp, sb.NT)) { sa.fuse_next = true; sa.resblock = true; sb.fused_prev = true; }
        }
    }
    // Whole stacks: a convolution with its fused pool followed by two fused residual blocks of the shapes the stack
    // kernel covers run as one launch (the tensors in between have no other reader by construction).
    if (!getenv("ACCERL_NO_STACK_FUSE")) {
        for (size_t si = 0; si + 5 < pol->steps.size(); ++si) {
            Step& sc = pol->steps[si];
            Step& sp = pol->steps[si + 1];
            Step& a1 = pol->steps[si + 2];
            Step& b1 = pol->steps[si + 3];
            Step& a2 = pol->steps[si + 4];
            Step& b2 = pol->steps[si + 5];
            if (sc.kind != ST_CONV || sc.el != EL_I8 || sc.pool_buf < 0 || sc.fuse_next || sc.fused_prev || sc.res_buf >= 0) continue;
            if (sp.kind != ST_MAXPOOL || !sp.fused || sp.out_buf != sc.pool_buf) continue;
            if (!(a1.kind == ST_CONV && a1.fuse_next && a1.resblock && b1.kind == ST_CONV && b1.fused_prev)) continue;
            if (!(a2.kind == ST_CONV && a2.fuse_next && a2.resblock && b2.kind == ST_CONV && b2.fused_prev)) continue;
            if (a1.in_buf != sc.pool_buf || a2.in_buf != b1.out_buf) continue;
            bool read_elsewhere = false;             // the pooled image and the first block's output feed the blocks only
            for (size_t sj = si + 6; sj < pol->steps.size(); ++sj)
                for (int b : {sc.pool_buf, b1.out_buf})
                    if (pol->steps[sj].in_buf == b || pol->steps[sj].res_buf == b) read_elsewhere = true;
            if (read_elsewhere) continue;
            if (!stack_supported(sc.cp, sc.NT, a1.cp, b1.cp, a2.cp, b2.cp)) continue;
            sc.stack_head = true;
            sp.stack_member = a1.stack_member = b1.stack_member = a2.stack_member = b2.stack_member = true;
        }
    }
    // The last convolution hands its output to the dense layer in the dense layer's MFMA fragment order when
    // nothing else reads that buffer: the dense kernel's state loads are then contiguous (row-major rows make
    // every lane of a quarter wavefront touch a different row).  Debug calls keep the plain layout.
    if (!getenv("ACCERL_NO_FRAG_HANDOFF")) {
        for (size_t gi = 0; gi < pol->steps.size(); ++gi) {
            Step& sg = pol->steps[gi];
            if (sg.kind != ST_GEMM || sg.el != EL_I8 || sg.epi != EPI_REQUANT || sg.in_buf < 0) continue;
            if (sg.gp.Kp_bytes != sg.gp.k_steps * 64) continue;
            int writer = -1, readers = 0;
            for (size_t sj = 0; sj < pol->steps.size(); ++sj) {
                const Step& t = pol->steps[sj];
                if (t.out_buf == sg.in_buf || t.pool_buf == sg.in_buf) writer = writer < 0 ? (int)sj : -2;
                if (t.in_buf == sg.in_buf || t.res_buf == sg.in_buf) ++readers;
            }
            if (writer < 0 || readers != 1) continue;
            Step& sc = pol->steps[writer];
            if (sc.kind != ST_CONV || sc.el != EL_I8 || sc.out_buf != sg.in_buf || sc.fused_prev || sc.fuse_next) continue;
            if (sc.res_buf >= 0 || sc.cp.pool || sc.cp.n_bands != 1 || sc.cp.sx != sc.cp.s) continue;
            const int cs = sc.cp.Cs_out;                                   // a pixel's channels must not straddle 16-byte blocks
            if (cs != 4 && cs != 8 && cs != 16 && cs != 32 && cs != 64) continue;
            if ((int64_t)sc.cp.Ho * sc.cp.Wo * sc.cp.Cs_out != sg.gp.Kp_bytes || sc.cp.G >= 2048) continue;
            sc.cp.out_frag = 1; sc.cp.frag_ks = sg.gp.k_steps;
            sg.gp.x_frag = 1;
        }
    }
    assign_slots(pol, 0);
    assign_slots(pol, 1);
    pol->ws_per_state = 0;
    for (const int64_t sz : pol->slots[0]) pol->ws_per_state += sz;
    // states per pass: about 1 GiB of intermediates, so that every launch still fills the chip
    pol->chunk = 0;
    if (pol->ws_per_state > 0) {
        int64_t ch = (1ll << 30) / pol->ws_per_state;
        if (ch < 1024) ch = 1024;
        if (ch > 16384) ch = 16384;
        pol->chunk = ch;
    }
    if (const char* env = getenv("ACCERL_CHUNK")) { const long v = atol(env); if (v > 0) pol->chunk = v < 65535 ? v : 65535; }
    // whole tiles of 64 states per pass: every pass after the first then starts on a 16-byte boundary of the uniforms,
    // values and actions, and on a tile boundary of the buffers handed over in fragment order
    if (pol->chunk > 0) pol->chunk = pol->chunk < 64 ? 64 : pol->chunk / 64 * 64;
    return ACCERL_OK;
}

int accerl_policy_create(const accerl_arch* arch, const void* weights, int64_t weights_bytes,
                         const float* quant_scales, int64_t n_scales, accerl_policy** out) {
    if (!out) return fail(ACCERL_EINVAL, "out is NULL");
    *out = nullptr;
    accerl_policy* pol = new (std::nothrow) accerl_policy();
    if (!pol) return fail(ACCERL_ENOMEM, "host allocation failed");
    std::vector<char> cst;
    int rc = create_host(arch, weights, weights_bytes, quant_scales, n_scales, pol, cst);
    if (rc) { delete pol; return rc; }
    hipError_t e = hipGetDevice(&pol->device);
    if (e == hipSuccess) e = hipMalloc((void**)&pol->consts, cst.size() + 256);
    if (e == hipSuccess) e = hipMemcpy(pol->consts, cst.data(), cst.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        rc = fail(e == hipErrorOutOfMemory ? ACCERL_ENOMEM : ACCERL_EHIP, "uploading constants: %s", hipGetErrorString(e));
        (void)hipGetLastError();
        if (pol->consts) (void)hipFree(pol->consts);
        delete pol;
        return rc;
    }
    *out = pol;
    return ACCERL_OK;
}

int accerl_plan_describe(const accerl_arch* arch, const void* weights, int64_t weights_bytes,
                         const float* quant_scales, int64_t n_scales, char* text, int64_t cap) {
    if (!text || cap < 1) return fail(ACCERL_EINVAL, "text buffer is NULL or empty");
    accerl_policy pol;
    std::vector<char> cst;
    int rc = create_host(arch, weights, weights_bytes, quant_scales, n_scales, &pol, cst);
    if (rc) return rc;
    std::string out;
    char line[512];
    static const char* kinds[] = {"mlp_fused", "quant_obs", "conv", "gemm", "gemm_f32", "maxpool", "lstm_pack", "sample", "heads"};
    snprintf(line, sizeof line, "steps=%d const_bytes=%lld ws_bytes_per_state=%lld chunk=%lld\n", (int)pol.steps.size(),
             (long long)cst.size(), (long long)pol.ws_per_state, (long long)pol.chunk);
    out += line;
    for (size_t i = 0; i < pol.steps.size(); ++i) {
        const Step& s = pol.steps[i];
        if (s.kind == ST_CONV) {
            const ConvParams& c = s.cp;
            const long lds = (s.KS > 0 ? 0 : c.w_bytes + c.k_steps * 16 + CONV_LDS_CONST) + (long)c.lds_tiles + (c.pool ? c.lds_otile : 0) + c.lds_tab;
            snprintf(line, sizeof line,
                     "step %zu conv layer=%d sub=%d el=%d in=%dx%dx%d out=%dx%dx%d k=%d s=%d pad=%d mode=%d NT=%d KS=%d "
                     "k_steps=%d RD=%d PF=%d TH=%d bands=%d G=%d units_img=%d pitch=%d tile_stride=%d lds=%ld wp=%d pt=%d pool=%d TPH=%d fuse_next=%d "
                     "front=%d tail=%d out_frag=%d resblock=%d pos23=%d stack=%d\n",
                     i, s.layer, s.sub, (int)s.el, c.H, c.W, c.Cs_in, c.Ho, c.Wo, c.Cs_out, c.k, c.s, c.pad, c.mode,
                     s.NT, s.KS, c.k_steps, s.RD, s.PF, c.TH, c.n_bands, c.G, c.units_img, c.pitch, c.tile_stride, lds, c.wave_private, c.wp_pt, c.pool, c.TPH, (int)s.fuse_next,
                     (int)(s.fuse_next && i + 1 < pol.steps.size() && conv_front_supported(c, s.NT, pol.steps[i + 1].cp)),
                     (int)(s.el == EL_I8 && !s.fused_prev && conv_tail_supported(c, s.NT)), c.out_frag, (int)s.resblock, c.pos23, s.stack_head ? 1 : s.stack_member ? 2 : 0);
        } else if (s.kind == ST_GEMM) {
            snprintf(line, sizeof line, "step %zu gemm layer=%d el=%d epi=%d N=%d Np=%d Kp_bytes=%d k_steps=%d n_tiles=%d relu_in=%d relu=%d x_frag=%d\n",
                     i, s.layer, (int)s.el, (int)s.epi, s.gp.N, s.gp.Np, s.gp.Kp_bytes, s.gp.k_steps, s.gp.n_tiles, s.gp.relu_in, s.gp.relu, s.gp.x_frag);
        } else {
            snprintf(line, sizeof line, "step %zu %s layer=%d\n", i, kinds[s.kind], s.layer);
        }
        out += line;
    }
    snprintf(text, (size_t)cap, "%s", out.c_str());
    return ACCERL_OK;
}

void accerl_policy_destroy(accerl_policy* p) {
    if (!p) return;
    for (auto& ev : p->events) (void)hipEventDestroy(ev.b);
    for (auto& ev : p->ev_starts) (void)hipEventDestroy(ev);
    if (p->ws) (void)hipFree(p->ws);
    if (p->consts) (void)hipFree(p->consts);
    if (p->mix_dev) (void)hipFree(p->mix_dev);
    for (int i = 0; i < 4; ++i) {
        if (p->mix_pin[i]) (void)hipHostFree(p->mix_pin[i]);
        if (p->mix_ev[i]) (void)hipEventDestroy(p->mix_ev[i]);
    }
    delete p;
}

static int forward_impl(accerl_policy* p, bool want_student, const void* states, int64_t B, const float* uniforms,
                        float* out_logits, float* out_value, int32_t* out_action, void* stream) {
    int rc = check_common(p, states, B, true, uniforms, out_logits, out_value, out_action);
    if (rc) return rc;
    if (want_student != (p->arch.precision == ACCERL_INT8))
        return fail(ACCERL_EINVAL, want_student ? "accerl_actor_forward needs an int8 policy" : "accerl_actor_forward_teacher needs an fp32 or bf16 policy");
    if (p->recurrent) return fail(ACCERL_EINVAL, "recurrent policy: use accerl_actor_forward_recurrent");
    Call c{states, B, uniforms, nullptr, nullptr, nullptr, out_logits, out_value, out_action, (hipStream_t)stream};
    return run(p, c);
}

int accerl_actor_forward(accerl_policy* p, const void* states, int64_t B, const float* uniforms,
                         float* out_logits, float* out_value, int32_t* out_action, void* stream) {
    return forward_impl(p, true, states, B, uniforms, out_logits, out_value, out_action, stream);
}

int accerl_actor_forward_teacher(accerl_policy* p, const void* states, int64_t B, const float* uniforms,
                                 float* out_logits, float* out_value, int32_t* out_action, void* stream) {
    return forward_impl(p, false, states, B, uniforms, out_logits, out_value, out_action, stream);
}

double accerl_mixture_alpha(double kl_mean, double kl_lo, double kl_hi) {
    if (kl_mean <= kl_lo) return 1.0;
    if (kl_mean >= kl_hi) return 0.0;
    return (kl_hi - kl_mean) / (kl_hi - kl_lo);
}

int accerl_actor_forward_mixture(accerl_policy* smaller, accerl_policy* original, const void* states, int64_t B,
                                 const float* uniforms, const uint8_t* use_smaller,
                                 float* out_logits, float* out_value, int32_t* out_action, void* stream) {
    int rc = check_common(smaller, states, B, true, uniforms, out_logits, out_value, out_action);
    if (rc) return rc;
    rc = check_common(original, states, B, true, uniforms, out_logits, out_value, out_action);
    if (rc) return rc;
    if (smaller->recurrent || original->recurrent) return fail(ACCERL_EUNSUPPORTED, "mixture of recurrent policies");
    const accerl_arch &as = smaller->arch, &ao = original->arch;
    if (as.obs_dtype != ao.obs_dtype || as.obs_c != ao.obs_c || as.obs_h != ao.obs_h || as.obs_w != ao.obs_w || as.n_actions != ao.n_actions)
        return fail(ACCERL_EINVAL, "the two policies differ in observation shape or number of actions");
    if (B == 0) return ACCERL_OK;
    if (!use_smaller) return fail(ACCERL_EINVAL, "use_smaller is NULL");
    if (B > 0x7fffffff) return fail(ACCERL_EINVAL, "batch too large for 32-bit row lists");
    hipStream_t st = (hipStream_t)stream;
    int64_t ns = 0;
    for (int64_t b = 0; b < B; ++b) ns += use_smaller[b] ? 1 : 0;
    const int64_t no = B - ns;
    if (no == 0 || ns == 0) {     // one network takes every row: no compaction needed
        Call c{states, B, uniforms, nullptr, nullptr, nullptr, out_logits, out_value, out_action, st};
        return run(ns ? smaller : original, c);
    }
    accerl_policy* m = smaller;
    const int A = as.n_actions;
    const int64_t obs = smaller->obs_bytes;
    if (obs % 16) return fail(ACCERL_EUNSUPPORTED, "mixture needs observation rows that are a multiple of 16 bytes");
    // ---- row lists through a pinned slot (the copy is asynchronous; a slot is reused only after its copy has finished)
    if (m->mix_pin_rows < B) {
        HIP_TRY(hipStreamSynchronize(st));
        for (int i = 0; i < 4; ++i) {
            if (m->mix_pin[i]) { HIP_TRY(hipHostFree(m->mix_pin[i])); m->mix_pin[i] = nullptr; }
            HIP_TRY(hipHostMalloc((void**)&m->mix_pin[i], (size_t)B * sizeof(int32_t), hipHostMallocDefault));
            if (!m->mix_ev[i]) HIP_TRY(hipEventCreateWithFlags(&m->mix_ev[i], hipEventDisableTiming));
        }
        m->mix_pin_rows = B;
    }
    auto rup = [](int64_t v) { return (v + 255) / 256 * 256; };
    const int64_t per_row = obs + 4 + 4 * (int64_t)A + 4 + 4;
    if (m->mix_rows < B) {
        HIP_TRY(hipStreamSynchronize(st));
        if (m->mix_dev) { HIP_TRY(hipFree(m->mix_dev)); m->mix_dev = nullptr; m->mix_rows = 0; }
        hipError_t e = hipMalloc((void**)&m->mix_dev, (size_t)(rup((B + 4) * 4) + rup((B + 4) * obs) + 4 * rup((B + 4) * 4 * (int64_t)(A > 1 ? A : 1)) + 4096));
        if (e != hipSuccess) { (void)hipGetLastError(); return fail(ACCERL_ENOMEM, "mixture workspace of %lld rows x %lld bytes", (long long)B, (long long)per_row); }
        m->mix_rows = B;
    }
    const int slot = m->mix_slot;
    m->mix_slot = (slot + 1) & 3;
    HIP_TRY(hipEventSynchronize(m->mix_ev[slot]));
    int32_t* pin = m->mix_pin[slot];
    {   // rows of the smaller policy first, then the original's, each in increasing order
        int64_t is = 0, io = ns;
        for (int64_t b = 0; b < B; ++b) { if (use_smaller[b]) pin[is++] = (int32_t)b; else pin[io++] = (int32_t)b; }
    }
    const int64_t cap = m->mix_rows + 4;         // the second subset starts at a row count rounded up to 4
    char* d = m->mix_dev;
    int32_t* d_idx = (int32_t*)d;               d += rup(cap * 4);
    char* d_states = d;                          d += rup(cap * obs);
    float* d_uni = (float*)d;                    d += rup(cap * 4);
    float* d_logits = (float*)d;                 d += rup(cap * 4 * (int64_t)A);
    float* d_value = (float*)d;                  d += rup(cap * 4);
    int32_t* d_action = (int32_t*)d;
    const int64_t o2 = (ns + 3) & ~(int64_t)3;   // keeps every buffer of the second subset 16-byte aligned
    HIP_TRY(hipMemcpyAsync(d_idx, pin, (size_t)B * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipEventRecord(m->mix_ev[slot], st));
    HIP_TRY(launch_gather_rows(states, d_idx, ns, obs, d_states, st));
    HIP_TRY(launch_gather_rows(states, d_idx + ns, no, obs, d_states + o2 * obs, st));
    HIP_TRY(launch_gather_f32(uniforms, d_idx, ns, d_uni, st));
    HIP_TRY(launch_gather_f32(uniforms, d_idx + ns, no, d_uni + o2, st));
    Call cs{d_states, ns, d_uni, nullptr, nullptr, nullptr, d_logits, d_value, d_action, st};
    rc = run(smaller, cs);
    if (rc) return rc;
    Call co{d_states + o2 * obs, no, d_uni + o2, nullptr, nullptr, nullptr, d_logits + o2 * A, d_value + o2, d_action + o2, st};
    rc = run(original, co);
    if (rc) return rc;
    HIP_TRY(launch_scatter_out(d_logits, d_value, d_action, d_idx, ns, A, out_logits, out_value, out_action, st));
    HIP_TRY(launch_scatter_out(d_logits + o2 * A, d_value + o2, d_action + o2, d_idx + ns, no, A, out_logits, out_value, out_action, st));
    return ACCERL_OK;
}

int accerl_actor_forward_recurrent(accerl_policy* p, const void* states, int64_t B, const float* uniforms,
                                   const uint8_t* done, float* h, float* c,
                                   float* out_logits, float* out_value, int32_t* out_action, void* stream) {
    int rc = check_common(p, states, B, true, uniforms, out_logits, out_value, out_action);
    if (rc) return rc;
    if (!p->recurrent) return fail(ACCERL_EINVAL, "policy has no lstm layer");
    if (B == 0) return ACCERL_OK;
    if (!h || !c) return fail(ACCERL_EINVAL, "h or c is NULL");
    if (((uintptr_t)h | (uintptr_t)c) & 15) return fail(ACCERL_EINVAL, "h or c is not 16-byte aligned");
    Call cl{states, B, uniforms, done, h, c, out_logits, out_value, out_action, (hipStream_t)stream};
    return run(p, cl);
}

int accerl_actor_forward_debug(accerl_policy* p, const void* states, int64_t B, int32_t layer, int32_t tap,
                               void* out, int64_t out_bytes, void* stream) {
    int rc = check_common(p, states, B, false, nullptr, nullptr, nullptr, nullptr);
    if (rc) return rc;
    if (B == 0) return ACCERL_OK;
    if (!out) return fail(ACCERL_EINVAL, "out is NULL");
    if ((uintptr_t)out & 15) return fail(ACCERL_EINVAL, "out is not 16-byte aligned");
    if (tap < ACCERL_TAP_ACC || tap > ACCERL_TAP_ACT_A) return fail(ACCERL_EINVAL, "bad tap kind");
    if ((tap == ACCERL_TAP_ACC || tap == ACCERL_TAP_ACC_A) && p->arch.precision != ACCERL_INT8)
        return fail(ACCERL_EINVAL, "accumulator taps are student-only");
    if (p->recurrent && layer >= p->arch.n_layers - 1) return fail(ACCERL_EINVAL, "recurrent policies: taps before the lstm only");
    Call c{states, B, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, (hipStream_t)stream};
    c.debug = true; c.layer = layer; c.tap = tap; c.out = out; c.out_bytes = out_bytes;
    return run(p, c);
}

int accerl_profile_begin(accerl_policy* p) {
    if (!p) return fail(ACCERL_EINVAL, "policy is NULL");
    for (auto& ev : p->events) (void)hipEventDestroy(ev.b);
    for (auto& ev : p->ev_starts) (void)hipEventDestroy(ev);
    p->events.clear();
    p->ev_starts.clear();
    p->profiling = true;
    return ACCERL_OK;
}

int accerl_profile_end(accerl_policy* p, int32_t cap, int32_t* n_steps, float* total_ms, int64_t* launches,
                       int32_t* layer, int32_t* kind) {
    if (!p || !n_steps) return fail(ACCERL_EINVAL, "policy or n_steps is NULL");
    p->profiling = false;
    const int n = (int)p->steps.size();
    *n_steps = n;
    int rc = ACCERL_OK;
    if (cap < n || !total_ms || !launches || !layer || !kind) rc = fail(ACCERL_EINVAL, "profile arrays need %d entries", n);
    if (rc == ACCERL_OK) {
        for (int i = 0; i < n; ++i) { total_ms[i] = 0.f; launches[i] = 0; layer[i] = p->steps[i].layer; kind[i] = (int)p->steps[i].kind; }
        for (auto& ev : p->events) {
            float ms = 0.f;
            hipError_t e = hipEventSynchronize(ev.b);
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
            if (e != hipSuccess) { rc = fail(ACCERL_EHIP, "reading profile events: %s", hipGetErrorString(e)); break; }
            total_ms[ev.step] += ms;
            launches[ev.step] += 1;
        }
    }
    for (auto& ev : p->events) (void)hipEventDestroy(ev.b);
    for (auto& ev : p->ev_starts) (void)hipEventDestroy(ev);
    p->events.clear();
    p->ev_starts.clear();
    return rc;
}

const char* accerl_last_error(void) { return g_err.c_str(); }

}  // extern "C"
