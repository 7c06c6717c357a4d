// Internal launch interface between the translation units of the library.
// All activations here are channels-innermost frames: [F][H][W][C].
#pragma once
#include "common.h"

namespace tsm {

// Geometry of one (shift-fused) convolution over F = N*T frames.
struct ConvP {
    int F, T;            // frames in the batch, frames per clip
    int H, W, Cin;       // input frame
    int Ho, Wo, Cout;    // output frame
    int KT, KH, KW;      // temporal (1 or 3) and spatial taps
    int stride, pad;     // spatial; the temporal taps use stride 1, padding KT/2
    int fold;            // channels shifted each way on the input (0: none)
    // Elements between consecutive input pixels; 0 means Cin.  A smaller pitch makes the "channels" of a tap
    // overlap the following pixels: a convolution whose taps along W are folded into the channel dimension
    // (MFMA kernels with Cin % 64 == 0 only; the caller guarantees that every read stays inside the tensor).
    int pitch = 0;
    int pix_pitch() const { return pitch ? pitch : Cin; }
    long rows_in() const { return (long)F * H * W; }
    long rows_out() const { return (long)F * Ho * Wo; }
    int taps() const { return KT * KH * KW; }
    long K() const { return (long)taps() * Cin; }
};

// ---- shift.hip ----------------------------------------------------------------
int shift_launch(const void* x, void* y, int N, int T, int C, int H, int W, int fold, int es, int layout,
                 int dir, hipStream_t s);
int transpose_frames(const void* in, void* out, int F, int rows, int cols, int es, hipStream_t s);

// ---- direct.hip: plain kernels for any shape, fp32 or bf16 storage ---------------
// Weights in the ABI order [Cout][Cin][KT*KH*KW], element type T (dtype).
int conv_direct_fwd(const ConvP& p, int dtype, const void* x, const void* w, void* y, hipStream_t s);
// dx = S^T(conv^T(dy, w)) (+ addend if not null, same shape as dx).
int conv_direct_dgrad(const ConvP& p, int dtype, const void* dy, const void* w, void* dx, const void* addend,
                      hipStream_t s);
// dw fp32 [Cout][Cin][taps]; must be zeroed by the caller unless accumulating.
int conv_direct_wgrad(const ConvP& p, int dtype, const void* x, const void* dy, float* dw, hipStream_t s);

// ---- elementwise.hip -----------------------------------------------------------------
// Per-channel reductions are deterministic and atomic-free: every block of a
// reduction kernel writes one row of a `partial` buffer, fp32 [blocks][2*C]
// (first C: sum / sum dz, next C: sum of squares / sum dz*yhat); the small kernel that
// consumes the statistics adds the rows up in fp64.
int fill_zero(void* p, size_t bytes, hipStream_t s);
// Rows of `partial` written by channel_stats / relu_bn_bwd_reduce for this tensor.
int red_blocks(long rows, int C, int dtype);
int channel_stats(int dtype, const void* y, long rows, int C, float* partial, hipStream_t s);
struct BnVec {           // per-channel fp32 vectors of one BatchNorm, each [C]
    float *mean, *rstd, *scale, *shift;
};
// mean/rstd/scale=gamma*rstd/shift=beta-mean*scale from the partial rows; optional running stats update.
int bn_finalize(const float* partial, int nblocks, long rows, int C, const float* gamma, const float* beta,
                float eps, BnVec out, float* run_mean, float* run_var, float momentum, hipStream_t s);
int stats_to_float(const float* partial, int nblocks, int C, float* sum, float* sumsq, hipStream_t s);
// scale = gamma / sqrt(var + eps), shift = beta - mean * scale (BatchNorm with known statistics)
int bn_eval_vec(const float* gamma, const float* beta, const float* mean, const float* var, float eps, int C,
                float* scale, float* shift, hipStream_t s);
// z = relu(scale*y + shift)
int bn_relu_apply(int dtype, const void* y, long rows, int C, const float* scale, const float* shift, void* z,
                  hipStream_t s);
// out = relu(scale*y + shift + sc), sc = shortcut (scale_d == null) or scale_d*shortcut + shift_d
// out_bits (nullable; only where block_tail_writes_bits): one byte per eight channels, [rows][C/8], bit j set where
// channel 8*v + j of the stored output is positive -- the ReLU decisions, a sixteenth of the tensor, for the backward pass.
bool block_tail_writes_bits(int dtype, int C);
int block_tail_fwd(int dtype, const void* y, long rows, int C, const float* scale, const float* shift,
                   const void* shortcut, const float* scale_d, const float* shift_d, void* out, hipStream_t s,
                   uint8_t* out_bits = nullptr);
// dz = dout * [act > 0] (act == null: no mask) written to dz_out (may alias dout; null: not written); partial rows receive
// sum dz and sum dz*yhat with yhat = (y - mean)*rstd.  If y2 != null a second BatchNorm (projection
// shortcut) is reduced into partial2.
int relu_bn_bwd_reduce(int dtype, const void* dout, const void* act, const void* y, long rows, int C,
                       const float* mean, const float* rstd, void* dz_out, float* partial, const void* y2,
                       const float* mean2, const float* rstd2, float* partial2, hipStream_t s);
// coef fp32 [3*C] such that dy = coef[c]*dz + coef[C+c]*y + coef[2C+c]; also dgamma, dbeta (nullable).
int bn_bwd_coeffs(const float* partial, int nblocks, long rows, int C, const float* mean, const float* rstd,
                  const float* gamma, float* coef, float* dgamma, float* dbeta, hipStream_t s);
int bn_bwd_apply(int dtype, const void* dz, const void* y, long rows, int C, const float* coef, void* dy,
                 hipStream_t s);
// The same for two BatchNorms that share the upstream gradient dz, from one read of it: dy1 from (y1, coef1), dy2 from
// (y2, coef2).  No buffer may alias another.
int bn_bwd_apply2(int dtype, const void* dz, const void* y1, const float* coef1, void* dy1, const void* y2,
                  const float* coef2, void* dy2, long rows, int C, hipStream_t s);
// out = a + b
int add_tensors(int dtype, const void* a, const void* b, void* out, size_t n, hipStream_t s);
// dtype conversion / repacking of weights
// ABI [Cout][Cin][taps] (dtype) -> bf16 [Cout][taps][CinP], channels ci >= Cin zero
int pack_weights_fwd(int dtype, const void* w, bf16_t* out, int Cout, int Cin, int taps, int CinP, hipStream_t s);
// ABI [Cout][Cin][KT][KH][KW] -> bf16 [Cin][flipped taps][Cout]
int pack_weights_dgrad(int dtype, const void* w, bf16_t* out, int Cout, int Cin, int KT, int KH, int KW,
                       hipStream_t s);
// fp32 [Cout][taps][CinP] -> fp32 [Cout][Cin][taps] (+= if accumulate)
int unpack_wgrad(const float* packed, float* dw, int Cout, int Cin, int taps, int CinP, int accumulate,
                 hipStream_t s);

// ---- conv_mfma.hip: bf16 MFMA implicit GEMM, channels-innermost -------------------------
bool mfma_conv_supported(const ConvP& p);
// Blocks the forward kernel launches for p (= rows of its statistics partial buffer).
int conv_mfma_fwd_blocks(const ConvP& p);
// y = conv(S(x)); wp = bf16 [Cout][taps][Cin]; stats_partial (nullable), fp32 [conv_mfma_fwd_blocks(p)][2*Cout],
// receives per block the per-channel sum / sum of squares of the stored (rounded) output.
// Optional epilogue (nullable): the stored result is act(scale[c]*y + shift[c] + res) -- BatchNorm with known
// statistics, the shortcut and the ReLU folded into the convolution; only where conv_mfma_fwd_can_fuse(p).
struct FwdEpilogue {
    const float* scale;
    const float* shift;
    const bf16_t* res;   // nullable, shape of y
    int relu;
};
bool conv_mfma_fwd_can_fuse(const ConvP& p);
int conv_mfma_fwd(const ConvP& p, const bf16_t* x, const bf16_t* wp, bf16_t* y, float* stats_partial,
                  const FwdEpilogue* ep, hipStream_t s);
// The 3x3 convolution of a bottleneck and the 1x1 convolution behind it in one kernel, forward only, with both
// BatchNorms as known per-channel affine maps (inference): out = relu(sc3*conv1x1(relu(sc2*conv3x3(x) + sh2)) + sh3
// + res).  p2 / p3 describe the two convolutions; w2p / w3p are their packed forward weights.  The intermediate
// tensor stays on the chip.  Supported: 64 -> 64 -> 256 and 128 -> 128 -> 512 channels, stride 1 or 2 on the 3x3.
bool conv_mfma_fused_tail_supported(const ConvP& p2, const ConvP& p3);
int conv_mfma_fused_tail(const ConvP& p2, const ConvP& p3, const bf16_t* x, const bf16_t* w2p, const bf16_t* w3p,
                         const float* sc2, const float* sh2, const float* sc3, const float* sh3, const bf16_t* res,
                         bf16_t* out, hipStream_t s);
// Optional fusion into the data-gradient epilogue: dx is the gradient w.r.t. act = ReLU(BatchNorm(y)) (all
// [rows_in][Cin] bf16); it is stored already masked with act > 0, and `partial`, fp32
// [conv_mfma_dgrad_blocks(p)][2*Cin], receives per block the per-channel sums of dz and of dz*(y-mean)*rstd.
struct DgradFuse {
    const bf16_t* act;
    const bf16_t* y;
    const float* mean;
    const float* rstd;
    float* partial;
    // optional: the decisions act > 0 as bits ([rows][Cin/8], see block_tail_fwd); kernels that can read them
    // instead of `act`, which must still be given
    const uint8_t* act_bits = nullptr;
};
// Blocks the data-gradient kernel launches for p when it can fuse (rows of DgradFuse::partial); 0 when this
// layer's kernel cannot.
int conv_mfma_dgrad_blocks(const ConvP& p);
// dx = S^T(conv^T(dy)) + addend; wd = bf16 [Cin][flipped taps][Cout]; fuse nullable.
// addend_stride 1: addend has the shape of dx.  2 (only where conv_mfma_dgrad_compact_addend_ok(p)): addend is
// [F][ceil(H/2)][ceil(W/2)][Cin] and holds the values for the pixels of dx whose row and column are even; all other
// pixels get nothing added (the data gradient of a 1x1 stride-2 convolution, whose other entries are zero).
bool conv_mfma_dgrad_compact_addend_ok(const ConvP& p);
int conv_mfma_dgrad(const ConvP& p, const bf16_t* dy, const bf16_t* wd, bf16_t* dx, const bf16_t* addend,
                    const DgradFuse* fuse, hipStream_t s, int addend_stride = 1);
// dw fp32, accumulated with atomics: zero it first (or keep what is there to accumulate).
// packed: [Cout][taps][p.Cin] (contiguous atomics, the fast order when taps > 1);
// otherwise the ABI order [Cout][cin_real][taps].  Channels >= cin_real are padding and are not written.
// affine_y / affine_coef (both or neither; only where conv_mfma_wgrad_affine_ok(p)): `dy` then holds dz, the gradient
// in front of a BatchNorm backward, and the kernel forms dy = a*dz + b*affine_y + c per output channel while loading
// (coefficients [3][Cout] from bn_bwd_coeffs, result rounded to bf16 as bn_bwd_apply would store it): for a layer
// whose dy nothing else reads, that pass and its tensor disappear.
bool conv_mfma_wgrad_affine_ok(const ConvP& p);
int conv_mfma_wgrad(const ConvP& p, const bf16_t* x, const bf16_t* dy, float* dw, int cin_real, bool packed,
                    hipStream_t s, const bf16_t* affine_y = nullptr, const float* affine_coef = nullptr);

}  // namespace tsm
