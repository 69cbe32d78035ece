// Internal declarations shared by the C-ABI translation unit and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "accerl.h"

namespace accerl {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

enum Elem : int { EL_I8 = 0, EL_BF16 = 1, EL_F32 = 2 };

// records the thread's error message and returns `code`
int set_error(int code, const char* msg);

// ---------------------------------------------------------------- fused int8 MLP (wave per 16 rows)
constexpr int MLP_MAX_LAYERS = 4;   // hidden layers; the heads come on top
struct MlpParams {
    const float* obs;        // [B, D] fp32
    const float* uniforms;   // [B]
    float* logits;           // [B, A]
    float* value;            // [B]
    int32_t* action;         // [B]
    int64_t B;
    int D;                   // observation width (<= 64)
    int A;                   // actions
    int n_hidden;            // hidden layers, each padded to 64 units
    float inv_s0;
    const v4i* wfrag;        // A-operand fragments, layer after layer: [layer][n_tile][64 lanes]
    const int32_t* bias;     // [layer][64] integer bias (heads last)
    const float* mult;       // [layer][64] requant multiplier (heads: dequant d)
    int lo[MLP_MAX_LAYERS];  // lower clamp per hidden layer (0 = fused ReLU, -127 otherwise)
    int k32;                 // D <= 32: the first layer's fragments are laid out for the K = 32 MFMA (8 features per lane)
    int p23;                 // every hidden layer has the fused ReLU and accumulators below 2^23 whatever the input
    const float* cfma;       // [layer][64] -2^23 * mult (p23 only)
    // debug taps (NULL = off): accumulator / activation of layer tap_layer, [B, n] row-major
    int32_t* tap_acc;
    int8_t* tap_act;
    int tap_layer;           // -1 = quantized observation (tap_act only)
    int tap_n;               // logical width of the tapped tensor
};
hipError_t launch_mlp_i8(const MlpParams& p, hipStream_t s);

// ---------------------------------------------------------------- observation quantizer (generic path)
hipError_t launch_quant_obs(const float* obs, int64_t B, int D, int Dpad, float inv_s0, int8_t* out, hipStream_t s);

// ---------------------------------------------------------------- convolution (input tiles in LDS, MFMA)
enum ConvMode : int { CM_FLAT = 0, CM_ROWS = 1, CM_U8T = 2, CM_ROWSV = 3 };
struct ConvParams {
    const void* in;          // NHWC elements, or NCHW uint8 observations (mode U8T)
    void* out;               // NHWC elements [B, Ho, Wo, Cs_out]
    const void* res;         // residual stream, same shape as out (NULL = none)
    int32_t* tap_acc;        // int32 [B, Ho, Wo, Cs_out] (NULL = off)
    const void* wfrag;       // [k_step][n_tile][64 lanes][16 B]
    const void* bias;        // int32 (int8 path, zero-point correction folded in) or fp32, [NT*16]
    const float* mult;       // [NT*16] (int8 path)
    const uint16_t* lut;     // 256 bf16 values obs/255 (bf16 path with uint8 source)
    int64_t B;
    int H, W;                // input image
    int Cin_real;            // channels present in the source
    int Cs_in;               // stored channels per input pixel (multiple of 4)
    int Ho, Wo, Cs_out;
    int k, s, pad;           // kernel rows, vertical stride, padding
    int sx;                  // horizontal stride in input pixels (a multiple of s when output pixels are packed)
    int TH;                  // output rows per band
    int n_bands;
    int in_rows;             // (TH-1)*s + k
    int pitch;               // bytes per LDS input row
    int tile_stride;         // LDS bytes per image tile (multiple of 16)
    int lds_tiles;           // LDS bytes of all tiles (every wave's, if wave-private) plus read slack
    int wave_private;        // every wavefront owns its batches of G images and its own LDS region
    int wave_tiles;          // wave-private: LDS bytes per wavefront region
    int wp_pt;               // wave-private: pixel tiles per iteration
    int cpr;                 // 16-byte chunks per kernel row
    int k_steps;             // MFMA steps (4 chunks each)
    int w_bytes;             // bytes of wfrag
    int relu_in;             // max(x, 0) on load
    int relu;                // teacher: ReLU after bias; student: lower clamp 0
    int src_u8;              // source is uint8 observations
    int mode;                // ConvMode: how a tile is staged
    int G;                   // images staged and multiplied together
    int img_bytes;           // FLAT: contiguous bytes per image
    int units_img;           // 16-byte staging units per image tile
    int row_units;           // ROWS / U8T: units per tile row
    uint32_t magic_units, magic_rowunits;   // ceil(2^32/d) for d = units per image tile, units per tile row (0 for d = 1)
    float inv_wo, hinv_wo;   // 1/Wo and 0.5/Wo
    // fused 3x3 stride-2 pad-1 max-pool of the layer's output (pool = 0: plain store to out)
    int pool;
    void* pool_out;          // pooled image [B, PH, PW, pool_unit << pool_ush bytes]
    int PH, PW, TPH;         // pooled size, pooled rows per band (TH then is the most conv rows a band needs)
    int pool_W;              // conv output pixels per row as stored (before any pixel packing)
    int pool_unit, pool_ush; // bytes per pooling unit (8 or 16), log2 of units per stored pixel
    int lds_otile;           // LDS bytes for the conv rows of a batch
    int lds_tab;             // LDS bytes of the pixel table of a thin layer (0 = none)
    float inv_prow, hinv_prow;   // 1/d and 0.5/d for d = pooling units per pooled row
    float r;                 // residual ratio (int8 path)
    // output in the fragment order of the dense layer that reads it (see GemmParams::x_frag); int8, no pooling,
    // no residual, one band
    int out_frag;
    int frag_ks;             // MFMA steps of that dense layer (64 bytes of K each)
    // int8 layer with the fused ReLU whose accumulators are all below 2^23 whatever the input (worked out from the
    // weights when the plan is built): a kernel may then start its accumulators at bias + 0x4B000000, read the result's
    // bits as the float 2^23 + acc and requantize with one fused multiply-add (see requant_relu4_p23)
    int pos23;
};
// KS > 0: weights in registers, that many MFMA steps unrolled; KS = 0: weights in LDS, runtime loop.
// RD: alignment (16 / 8 / 4) of a chunk read in LDS.  PF: staging units per lane the kernel holds.
hipError_t launch_conv(const ConvParams& p, Elem el, int NT, int KS, int RD, int PF, hipStream_t s);
bool conv_pick_variant(Elem el, int NT, int k_steps, int RD, int mode, int pf, bool extras, int* KS, int* PF);
int conv_pixel_tiles(int NT);
constexpr int CONV_LDS_CONST = 512;   // LDS bytes for bias and multipliers in the LDS-weight kernels
bool conv_wp_available(Elem el, int NT, int RD, int PT, int units);
constexpr int CONV_WP_NWAVES = 8;

// first two int8 convolutions of an image policy in one kernel (the first layer's output stays in LDS)
bool conv_fused_supported(const ConvParams& a, int NTA, int KSA, int RDA, const ConvParams& b, int NTB, int KSB, int RDB);
hipError_t launch_conv_fused(const ConvParams& a, int NTA, const ConvParams& b, hipStream_t s);
// the same pair for exactly the paper's original network (84x84x4 -> 8x8/4 x32 -> 4x4/2 x64): sizes fixed at compile time
bool conv_front_supported(const ConvParams& a, int NTA, const ConvParams& b);
hipError_t launch_conv_front(const ConvParams& a, const ConvParams& b, hipStream_t s);
// a residual block (ReLU - conv3x3 - ReLU - conv3x3 + skip) of the pruned IMPALA student in one kernel: a = first, b = second convolution
bool resblock_supported(const ConvParams& a, int NTA, const ConvParams& b, int NTB);
hipError_t launch_resblock(const ConvParams& a, const ConvParams& b, hipStream_t s);
// a whole stack of the IMPALA-style student (conv3x3 + max-pool 3x3/2 + two residual blocks) in one kernel:
// c = the stack convolution planned with its fused pool, a1 / b1 and a2 / b2 = the two blocks' convolutions
bool stack_supported(const ConvParams& c, int NTC, const ConvParams& a1, const ConvParams& b1, const ConvParams& a2, const ConvParams& b2);
hipError_t launch_stack(const ConvParams& c, const ConvParams& a1, const ConvParams& b1, const ConvParams& a2, const ConvParams& b2, hipStream_t s);
// the third layer of that network (9x9x64 -> 3x3/1 x64) with sizes fixed at compile time
bool conv_tail_supported(const ConvParams& p, int NT);
hipError_t launch_conv_tail(const ConvParams& p, hipStream_t s);

// ---------------------------------------------------------------- max pooling on NHWC
hipError_t launch_maxpool(const void* in, void* out, int64_t B, int H, int W, int Cs, int Ho, int Wo,
                          int k, int s, int pad, Elem el, hipStream_t stream);

// ---------------------------------------------------------------- row gather / scatter (policy mixture)
hipError_t launch_gather_rows(const void* in, const int32_t* idx, int64_t n, int64_t row_bytes, void* out, hipStream_t s);
hipError_t launch_gather_f32(const float* in, const int32_t* idx, int64_t n, float* out, hipStream_t s);
hipError_t launch_scatter_out(const float* logits, const float* value, const int32_t* action, const int32_t* idx, int64_t n, int A,
                              float* out_logits, float* out_value, int32_t* out_action, hipStream_t s);

// ---------------------------------------------------------------- dense layers (MFMA GEMM)
enum GemmEpi : int { EPI_REQUANT = 0, EPI_HEADS_I8 = 1, EPI_BF16 = 2, EPI_HEADS_F32ACC = 3, EPI_LSTM = 4 };
struct GemmParams {
    const void* x;           // [B, Kp] elements (Kp = padded K, multiple of 16 bytes)
    const void* wfrag;       // [n_tiles][k_steps][64 lanes][16 B]
    const void* bias;        // int32 or fp32, [n_tiles*16]
    const float* mult;       // [n_tiles*16]
    void* out;               // EPI_REQUANT: int8 [B, Np]; EPI_BF16: bf16 [B, Np]
    int32_t* tap_acc;        // int32 [B, N] (NULL = off)
    float* logits;           // heads
    float* value;
    // LSTM epilogue
    float* h;                // [B, Hd] in/out
    float* c;
    int64_t B;
    int Kp_bytes;            // row pitch of x in bytes
    int k_steps;
    int N;                   // logical outputs
    int Np;                  // stored outputs per row (out pitch in elements)
    int n_tiles;
    int relu_in;
    int relu;
    int A;                   // heads: actions
    int Hd;                  // lstm hidden
    // x is stored in MFMA fragment order: [tile of 16 states][k_step][lane = 16 * (k % 64 / 16) + state % 16][16 B],
    // so that a wavefront's fragment load is one contiguous KiB (a row-major x makes every lane of a quarter
    // wavefront touch a different row).  Needs Kp_bytes == 64 * k_steps and storage for whole tiles of 16 states.
    int x_frag;
};
hipError_t launch_gemm(const GemmParams& p, Elem el, GemmEpi epi, hipStream_t s);
// int8 + requantizing epilogue for large batches whose rows are whole MFMA steps (launch_gemm picks it)
bool gemm_stream_supported(const GemmParams& p);
hipError_t launch_gemm_stream(const GemmParams& p, hipStream_t s);

// policy heads + sampler in one kernel (K up to 16 MFMA steps; wider inputs go through launch_gemm + launch_sample)
struct HeadsParams {
    const void* x;           // [B, Kp] elements
    const void* wfrag;       // [n_tiles][k_steps][64 lanes][16 B]
    const void* bias;        // int32 or fp32, [n_tiles*16]
    const float* mult;       // [n_tiles*16] dequantisation (int8)
    const float* uniforms;
    float* logits; float* value; int32_t* action;
    int32_t* tap_acc;        // int32 [B, A+1] (NULL = off)
    int64_t B;
    int Kp_bytes, k_steps, A, relu_in;
};
bool heads_supported(int k_steps, int Kp_bytes, int A);
hipError_t launch_heads(const HeadsParams& p, Elem el, hipStream_t s);

// fp32 dense layer (teacher MLP): out = relu?(x W^T + b); heads variant writes logits/value
struct GemmF32Params {
    const float* x; const float* w; const float* bias; float* out; float* logits; float* value;
    int64_t B; int K; int N; int ldx; int ldo; int relu; int heads; int A;
};
hipError_t launch_gemm_f32(const GemmF32Params& p, hipStream_t s);

// LSTM operand packing: xh[b] = [bf16(x[b]) , bf16(done ? 0 : h[b])], and h,c zeroed where done
struct LstmPackParams {
    const void* x; int x_elem; float x_scale; int x_pitch_bytes; int x_relu; int In;
    const uint8_t* done; float* h; float* c; uint16_t* xh; int Hd; int64_t B;
};
hipError_t launch_lstm_pack(const LstmPackParams& p, hipStream_t s);

// ---------------------------------------------------------------- sampler
hipError_t launch_sample(const float* logits, const float* uniforms, int32_t* action, int64_t B, int A, hipStream_t s);

// ---------------------------------------------------------------- debug conversions
hipError_t launch_bf16_to_f32(const uint16_t* in, float* out, int64_t n, hipStream_t s);

}  // namespace accerl
