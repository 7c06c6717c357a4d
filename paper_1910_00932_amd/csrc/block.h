// Internal description of one residual block (channels-innermost frames) shared
// by the block entry points and the TSM-ResNet-50 step.
#pragma once
#include "internal.h"

namespace tsm {

struct StageDef {
    ConvP p;
    const void* w;        // weights, ABI order [Cout][Cin][taps], block dtype
    const bf16_t* wp;     // optional pre-packed forward weights  [Cout][taps][Cin]
    const bf16_t* wd;     // optional pre-packed dgrad weights    [Cin][flipped taps][Cout]
    const float *g, *b;   // BatchNorm scale / offset
    float *dw, *dg, *db;  // gradients (fp32)
    float *run_mean, *run_var;  // optional running statistics
    float* dwp = nullptr;  // optional zeroed buffer [Cout][taps][Cin] that receives the weight gradient of a several-tap
                           // convolution in the packed order; the caller permutes it into dw afterwards
};

struct BlockPlan {
    int nst;              // 2 (basic) or 3 (bottleneck) convolution stages
    StageDef st[3];
    bool proj;
    StageDef ds;          // projection shortcut
    int dtype;
    float eps, bn_momentum;
    bool grads_prezeroed;  // the caller zeroed every dw: weight gradients are added without a fill
    // Chaining inside a network (both optional).  dout_part: the gradient handed to block_bwd_impl is already
    // masked with out > 0 and the BatchNorm sums of the last stage are in dout_part, dout_nb rows (the
    // producer was a fused data gradient).  dx_fuse: applied to the data gradient that produces dx.
    const float* dout_part;
    int dout_nb;
    bool dout_masked;      // the gradient handed to block_bwd_impl is already masked with out > 0, without sums (the
                           // producer was a data gradient in mask-only mode): the sums are reduced from it
    const DgradFuse* dx_fuse;
    // saved-for-backward buffers (caller-owned memory)
    void* y[3];           // convolution outputs
    void* z[2];           // ReLU(BN(y)) of all but the last stage
    void* yd;             // projection output
    BnVec bn[3], bnd;
    void *x_copy, *out_copy;  // channels-innermost copies when the caller's order is NTCHW
    uint8_t* out_bits = nullptr;  // optional: receives the ReLU decisions of the block's output (see block_tail_fwd)
};

int conv_stats_blocks(const ConvP& p, int dtype);
int run_conv_fwd(const ConvP& p, int dtype, const void* x, const void* w, const bf16_t* wp, void* y,
                 float* stats_partial, Arena& ws, bool dry, hipStream_t s);
// Rows of the partial buffer a fused data gradient fills (see DgradFuse); 0 when it cannot fuse.
int conv_dgrad_fuse_blocks(const ConvP& p, int dtype);
int run_conv_dgrad(const ConvP& p, int dtype, const void* dy, const void* w, const bf16_t* wd, void* dx,
                   const void* addend, const DgradFuse* fuse, Arena& ws, bool dry, hipStream_t s, int addend_stride = 1);
int run_conv_wgrad(const ConvP& p, int dtype, const void* x, const void* dy, float* dw, float* dwp, int accumulate, Arena& ws,
                   bool dry, hipStream_t s);

// Forward pass of one block with every BatchNorm as a known per-channel affine map (inference): per stage i
// (0..nst-1, 3 = projection) packed forward weights wp[i] (bf16 path, nullable: packed into the workspace then) and
// scale / shift vectors sc[i] / sh[i].  Buffers, all caller-owned: mid0 / mid1 hold the outputs of all but the last
// stage, ytmp a raw convolution output where the kernel cannot apply the map itself, scbuf the projection shortcut
// (ytmp and scbuf: size of the block's output).  On the bf16 path the maps, the shortcut and the ReLUs ride in the
// convolution epilogues, and the last two convolutions of a bottleneck run as one kernel where there is one.
struct InferParams {
    const bf16_t* wp[4];
    const float* sc[4];
    const float* sh[4];
};
int block_infer_impl(BlockPlan& b, const InferParams& ip, const void* x, void* out, void* mid0, void* mid1, void* ytmp,
                     void* scbuf, Arena& ws, bool dry, hipStream_t s);

int make_block_plan(const tsm_block_desc* d, BlockPlan* b, const char* who);
void block_saved_layout(BlockPlan& b, Arena& sv, bool keep_x_copy);
int block_fwd_impl(BlockPlan& b, const void* x, void* out, Arena& ws, bool dry, hipStream_t s);
// dx may be null (no input gradient wanted).
int block_bwd_impl(BlockPlan& b, const void* x, const void* out, const void* dout, void* dx, Arena& ws, bool dry,
                   hipStream_t s, int lag_slot = -1);
int block_bwd_flush(hipStream_t s);
// A branch of independent work on the library's second stream, forked behind what `s` holds so far; returns `s` itself
// where there is no second stream (one-stream mode, profiling).  side_branch_end joins it, on every path.
hipStream_t side_branch_begin(hipStream_t s);
int side_branch_end(hipStream_t s, hipStream_t branch);

}  // namespace tsm
