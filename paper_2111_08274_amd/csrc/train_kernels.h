// Kernel launchers of the local-training path (paper Sec. 2.1: forward, backward, update), all grouped over
// replicas: grid z (or y) indexes a slot g of the active prefix, and order[g] is the replica it works on.
#pragma once
#include "hadfl_internal.h"

namespace hadfl {

enum GemmMode { kFwd = 0, kDgrad = 1, kWgrad = 2 };

// One grouped implicit-GEMM launch C[M x N] = A[M x K] * B[K x N] per active replica.
//  kFwd   : M = B*Ho*Wo, N = Cout,   K = R*S*Cin   A = im2col(X),        B = W[(r,s,ci)][co]
//  kDgrad : M = B*H*W,   N = Cin,    K = R*S*Cout  A = col(dY),          B = W^T per tap
//  kWgrad : M = R*S*Cin (+1 bias row), N = Cout, K = B*Ho*Wo  A = im2col(X)^T, B = dY   (split over K)
// A dense layer is the 1x1 case with H = W = 1 and Cin = flattened input size.
struct GemmParams {
    int mode;
    int B, H, W, Cin, Ho, Wo, Cout, R, S, stride, pad;
    int M, N, K;
    int tiles_m, tiles_n;
    int grid_y, n_active;         // set by the fp32 launcher: splits (or dgrad pixel classes) and active replicas
    int kchunk, splits;
    int hw_shift, w_shift;        // log2 of Ho*Wo and Wo (kWgrad) when powers of two, else -1
    // activation-side source: X (fwd, wgrad) or dY (dgrad)
    const float* a; long long a_rep;
    const long long* cursor; int n_samples, batch; long long sample_sz;   // a is the data set when cursor != null
    const float* w; long long w_rep;              // weights of this layer inside the replica rows
    const float* dy; long long dy_rep;            // kWgrad: dY
    float* out; long long out_rep, out_split;     // kWgrad with splits > 1: partial sums [g][split][M*N]
    int has_bias, relu, accumulate;
    // kDgrad: when set, the written gradient is zeroed where mask <= 0 (mask = the ReLU output stored in the tensor
    // whose gradient is being produced, so the result is the gradient before that fused ReLU)
    const float* mask; long long mask_rep;
    int a_f32;                    // bf16 kernel only: the activation-side source is the fp32 data set
    const int* order;
};
hipError_t launch_gemm(const GemmParams& p, int n_active, hipStream_t s);
// Same problems with bf16 activations / activation gradients (pointers still typed float*: they are byte bases whose
// offsets and strides are counted in 4-byte units), fp32 weights rounded to bf16 on the fly, fp32 weight gradients.
hipError_t launch_gemm_bf16(const GemmParams& p, int n_active, hipStream_t s);
// out[rep][i] = sum_s partial[g][s][i], s ascending
hipError_t launch_splitk_reduce(const float* partial, long long split_stride, int splits, float* out, long long out_rep,
                                long long count, const int* order, int n_active, hipStream_t s);
// The same sum applied as the update of the layer's parameters (w, buf: first parameter of the layer in replica row 0;
// buf may be null).  Needs count, split_stride and row_stride multiples of 4 and 16-byte aligned pointers.
hipError_t launch_splitk_reduce_update(const float* partial, long long split_stride, int splits, float* w, float* buf,
                                       long long row_stride, long long count, float lr, float momentum, const int* order,
                                       int n_active, hipStream_t s);

// ---- lean bf16 kernels for regular stride-1 "same" convolutions (conv_bf16_fast.hip) ----
struct FastConvParams {      // out[m][n] = sum_k act[pixel(m) + tap(k)][c(k)] * wmat[n][k]; M = B*H*W, K = R*S*C
    int B, H, W, C, N, R, S, pad, M, K;
    const void* a; long long a_rep;            // bf16 activations (forward) or output gradient (data gradient)
    const __bf16* wmat; long long wmat_rep;    // bf16 [N][K], per-replica stride in elements
    void* out; long long out_rep;              // bf16 [M][N]
    const float* bias; long long bias_rep;     // forward: fp32 bias inside the replica rows, or null
    int relu;
    const void* mask; long long mask_rep; int accumulate;   // data gradient
    const int* order;
    int tile_hint;                             // 1: take the 256 x 256 tiles whenever the shape allows (N % 256 == 0)
    // optional position table (both null or both set): GEMM row ps * B + b is image b at pixel perm[ps]; posmask[ps] has
    // bit r * S + s set when tap (r, s) of that pixel lies inside the image
    const int* perm; const unsigned* posmask;
    int n_active;                              // set by the launcher
    // forward only, optional: per-channel sums of the stored outputs for the batch norm that follows.  Entry e of slot g
    // covers GEMM rows [e * R, (e + 1) * R), R = the chosen kernel's rows per tile (reported by the launcher):
    // stat[g * stat_rep + e * 2 * N + n] = sum of out[m][n], [.. + N + n] = sum of out[m][n]^2 (values as rounded to bf16)
    float* stat; long long stat_rep;
    // data gradient only, with stat set: the tensor whose gradient is being written is the output y of a batch norm
    // (after its fused ReLU and, if the pool is folded into it, after the pool), and the same entries receive what that
    // batch norm's backward pass needs instead:  [..+ n] = sum of g,  [.. + N + n] = sum of g * y,  g the stored gradient
    // (zero where stat_relu is set and y <= 0).  With xhat = (y - beta) / gamma wherever the gradient passes, these give
    // d(beta) = sum g and d(gamma) = (sum g*y - beta * sum g) / gamma without another pass over the tensors.
    const void* stat_y; long long stat_y_rep; int stat_relu;
};
// epi 0: forward (+bias, ReLU); epi 1: data gradient (mask, accumulate).  Needs C % 64 == 0 and N % 64 == 0.
// stat_rows (may be null): receives the rows per statistics entry of the kernel that was launched (128 or 256).
hipError_t launch_conv_fast(const FastConvParams& p, int epi, int n_active, hipStream_t s, int* stat_rows = nullptr);

struct FastWgradParams {     // dW[(tap, ci) | bias row][co] over pixels; needs C % 8 == 0, N % 64 == 0, H, W powers of two
    int B, H, W, C, N, R, S, pad, M, K, kchunk, splits, w_shift, has_bias;
    const void* x; long long x_rep;
    const void* dy; long long dy_rep;
    float* out; long long out_rep, out_split;
    const int* order;
    const int* perm; const unsigned* posmask;   // optional position table as in FastConvParams; needs B % 64 == 0, kchunk % 64 == 0
    int tile_hint;                              // 1: 256-row tiles whenever N % 128 == 0
    // splits == 1 only: when sgd_w is set the epilogue applies the update (buf = momentum*buf + g; w -= lr*buf) to the
    // layer's slice of the parameter rows (same per-replica stride as `out`) instead of storing the gradient
    float* sgd_w; float* sgd_buf; float lr, momentum;
    int n_active;                               // set by the launcher
};
hipError_t launch_wgrad_fast(const FastWgradParams& p, int n_active, hipStream_t s);

// ---- bf16 configuration, first convolution (fp32 data set in, few channels): conv_first_bf16.hip ----
struct FirstConvParams {     // K = R*S*C footprint values per pixel (K + bias row <= 32), N = 32 or 64 output channels, stride 1
    const float* x; const long long* cursor; int n_samples;     // data set [replica][n_samples][H][W][C] and batch cursors
    int B, H, W, C, N, R, S, pad, K, M;                          // M = B*H*W pixels of a batch
    const float* w; long long w_rep;                             // fp32 weights [K][N] inside the replica rows (stride w_rep)
    const float* bias;                                           // inside the same rows, or null
    void* out; long long out_rep; int relu;                      // forward: bf16 [M][N]
    const void* dy; long long dy_rep;                            // weight gradient: bf16 [M][N]
    float* gout; long long gout_rep, gout_split; int splits, kchunk;   // rows 0..K-1 weights, row K bias; split over pixels
    const int* order;
};
bool conv_first_supported(const FirstConvParams& p);
hipError_t launch_conv_first_fwd(const FirstConvParams& p, int n_active, hipStream_t s);
hipError_t launch_conv_first_wgrad(const FirstConvParams& p, int n_active, hipStream_t s);

struct WeightPrepParams {    // fp32 W[tap][C][N] -> bf16 Wf[N][tap*C + ci] and Wb[C][(taps-1-tap)*N + co]
    const float* w; long long w_rep;
    __bf16* wf; __bf16* wb; long long wbf_rep;
    int C, N, taps;
    const int* order;
};
hipError_t launch_weight_prep(const WeightPrepParams& p, int n_active, hipStream_t s);

// fp32 configuration: the same kernel plan in fp32 (conv_f32_fast.hip).  FastConvParams with a, wmat, out, mask pointing at
// floats (wmat_rep in floats); needs C % 32 == 0, N % 64 == 0.  stat / stat_rows as in launch_conv_fast.
hipError_t launch_conv_f32_fast(const FastConvParams& p, int epi, int n_active, hipStream_t s, int* stat_rows = nullptr);
struct WeightPrepF32Params {    // fp32 W[tap][C][N] -> fp32 Wf[N][tap*C + ci] and Wb[C][(taps-1-tap)*N + co]
    const float* w; long long w_rep;
    float* wf; float* wb; long long wcopy_rep;
    int C, N, taps;
    const int* order;
};
hipError_t launch_weight_prep_f32(const WeightPrepF32Params& p, int n_active, hipStream_t s);

struct DenseSmallParams {     // out[m][n] = sum_k x[m][k] w[k][n] + bias[n], N <= 16
    const float* x; long long x_rep;
    const float* w; long long w_rep;     // weights [K][N] followed by bias [N]
    float* out; long long out_rep;
    int rows, K, N, has_bias;
    int bf16;
    const int* order;
};
hipError_t launch_dense_small_fwd(const DenseSmallParams& p, int n_active, hipStream_t s);

struct EwParams {     // element-wise / pooling kernels
    const float* in; long long in_rep;
    const float* in2; long long in2_rep;
    float* out; long long out_rep;
    long long count;              // elements per replica of `out`
    int B, H, W, C;               // input geometry where needed
    int accumulate;
    int relu;                     // forward kernels: apply max(., 0) to the result
    const float* mask; long long mask_rep;   // backward kernels: zero the written gradient where mask <= 0
    int bf16;                     // tensors are bf16 (strides still in 4-byte units)
    const int* order;
};
hipError_t launch_relu_fwd(const EwParams& p, int n_active, hipStream_t s);
// out(din) (+)= in2(dout) where in(x) > 0
hipError_t launch_relu_bwd(const EwParams& p, int n_active, hipStream_t s);
hipError_t launch_maxpool_fwd(const EwParams& p, int n_active, hipStream_t s);
// in = pool input x, in2 = dout (pooled shape), out = din (input shape)
hipError_t launch_maxpool_bwd(const EwParams& p, int n_active, hipStream_t s);
hipError_t launch_add_fwd(const EwParams& p, int n_active, hipStream_t s);
// out(din) (+)= in(dout)
hipError_t launch_pass_grad(const EwParams& p, int n_active, hipStream_t s);
hipError_t launch_gap_fwd(const EwParams& p, int n_active, hipStream_t s);
hipError_t launch_gap_bwd(const EwParams& p, int n_active, hipStream_t s);

struct BnParams {
    const float* x; long long x_rep;       // [rows][C]
    float* y; long long y_rep;             // forward output / backward dx
    const float* dy; long long dy_rep;
    float* params; long long row_stride;   // replica rows; gamma at w_off, beta at w_off + C, running stats at stat_off
    float* grads;                          // gradient rows (same layout)
    long long w_off, stat_off;
    float* saved; long long saved_rep;     // [2][C]: mean, 1/sqrt(var+eps)
    float* partial; long long partial_rep; // [chunks][2][C]
    int rows, C, chunks, chunk_rows;
    int cvb;                               // set by the launcher: channel vectors per workgroup (vector kernels)
    int accumulate;
    int relu;                              // forward: y = max(bn(x), 0)
    const float* mask; long long mask_rep; // backward: zero dx where mask <= 0
    int bf16;
    const int* order;
    // a 2x2 / stride-2 max-pool folded into the layer (vector kernels only; H, W even): forward writes the pooled
    // output only; backward takes the gradient of the pooled output instead of dy and forms each window's outputs
    // again from x
    int pool, H, W;
    // forward: the producing convolution already left per-entry sums of d = x - x0 and d^2 in `partial`
    // ([stat_entries][2][C]) and the sums pass is skipped; the shift x0 of channel c is that convolution's bias
    // stat_shift[c] (zero without one): what the outputs are centred on when the bias is large beside their spread
    int stats_done, stat_entries;
    const float* stat_shift; long long stat_shift_rep;
    // backward: the data-gradient kernel of the layer above already left per-entry sums of g and g * y in `partial`
    // ([stat_entries][2][C], see FastConvParams::stat_y); the sums pass is skipped and d(gamma) is formed from them
    int bwd_stats_done;
    float* pool_out; long long pool_out_rep;
    const float* pool_g; long long pool_g_rep;
};
hipError_t launch_bn_fwd(const BnParams& p, int n_active, hipStream_t s);
hipError_t launch_bn_bwd(const BnParams& p, int n_active, hipStream_t s);

struct LossParams {
    const float* logits; long long logits_rep;
    float* dlogits; long long dlogits_rep;
    const int* y; const long long* cursor; int n_samples, batch, n_classes;
    float* loss;
    int bf16;
    const int* order;
};
hipError_t launch_softmax_ce(const LossParams& p, int n_active, hipStream_t s);

constexpr int kMaxSgdSegments = 16;
struct SgdParams {
    float* w; const float* g; float* buf; long long row_stride;
    float lr, momentum;
    long long* cursor; int* versions;      // bumped once per replica per step (when bump is set)
    int bump;
    // the launch covers n_seg pieces of each row: floats [first[k], first[k] + count[k]), all multiples of 4
    int n_seg; long long first[kMaxSgdSegments], count[kMaxSgdSegments];
    const int* order;
};
hipError_t launch_sgd(const SgdParams& p, int n_active, hipStream_t s);

}  // namespace hadfl
