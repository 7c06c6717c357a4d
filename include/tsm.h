/*
 * tsm.h -- C ABI of the MI355X (gfx950) hot path of TSM video training.
 *
 * The operator and the network come from "Training Kinetics in 15 Minutes"
 * (arXiv 1910.00932): the Temporal Shift Module (section 2, "Temporal modeling
 * unit", Fig. 1) inserted into every residual block of a 2-D ResNet-50
 * (section 3, model (3); Table 2: 8 frames at every stage), trained with
 * synchronous SGD (section 4.1).  This library is the single-GPU part of one
 * training iteration: shift, shift-fused convolutions with their two gradients,
 * BatchNorm/ReLU, residual blocks, and the whole TSM-ResNet-50 step.
 *
 * Conventions for every entry point
 *  - Every data pointer is DEVICE memory owned by the caller unless a comment
 *    says "host".  The library allocates no device memory; scratch space comes in
 *    through the (ws, ws_bytes) pair, sized by the matching *_workspace_bytes().
 *  - Calls are asynchronous on the caller's hipStream_t (passed as void*; NULL is
 *    the default stream) and never synchronise the device.  The training entry
 *    points (tsm_block_fwd, tsm_block_bwd, tsm_resnet50_step,
 *    tsm_resnet50_accum_step) run the weight gradients and the kernels of a
 *    projection shortcut on a second stream that the library creates per host thread
 *    and device on first use; it forks from and joins the caller's stream with
 *    events inside the call, so the call as a whole stays ordered on the caller's
 *    stream and can be recorded into a HIP graph (make the first call on a device
 *    outside stream capture).  TSM_WGRAD_OVERLAP=0 in the environment keeps
 *    everything on the caller's stream.
 *  - Which kernel runs a convolution is the library's choice and does not change
 *    what is computed.  For comparisons the environment can take choices away:
 *    TSM_IGEMM_RING=0 / TSM_WGRAD_TR=0 (read once per process) fall back to the
 *    kernels for channel counts that are not multiples of 64 wherever those can
 *    run; TSM_CONV3X3_C64=0 and TSM_STEM_KERNEL=0 (read at every call) leave the
 *    layers that have a kernel of their own to the general one (TSM_STEM_PW=0,
 *    read at every call, keeps the stem on the block-wide one of its two
 *    kernels), and
 *    TSM_CONV3X3_C64_MIN_TILES=<n> (read at every call) replaces the number of
 *    256-pixel tiles from which those two kernels are chosen (default: five per
 *    compute unit); TSM_IGEMM_BM=128|256 (read once per process) fixes the rows
 *    per tile of the general forward / data-gradient kernel, which otherwise
 *    follows from the number of tiles per compute unit; TSM_IGEMM_WIDE=0 (read at
 *    every call) keeps 128-column tiles for the forward layers that would run on
 *    256-column tiles (results that are a multiple of 256 channels wide,
 *    statistics epilogue, from half a round of such tiles on:
 *    TSM_IGEMM_WIDE_MIN_TILES=<n> replaces that number); TSM_IGEMM_NARROW=0 (read once
 *    per process) keeps 128-column tiles where the library would take 64
 *    columns to fill the machine; TSM_FUSED_TAIL=0 (read
 *    at every call) keeps the inference paths on one kernel per convolution and
 *    TSM_FUSED_TAIL_MIN_TILES=<n> replaces the number of 256-pixel tiles from
 *    which the two-convolution kernel is chosen (default: three per four
 *    compute units); TSM_PW_KERNEL=0 (read at every call) leaves the short-K 1x1
 *    layers that have kernels of their own (64, 128 or 256 channels into a result
 *    at least twice as wide, up to 1024 channels: forward, and the data gradient
 *    of a block's first convolution) to the
 *    general kernel and TSM_PW_MIN_ROWS=<n> replaces the number of pixels from
 *    which their own kernel is chosen (default: one pass of 32 pixels per
 *    wavefront of the grid); TSM_WGRAD_XCD=0 (read at every call) launches the
 *    weight gradient's tiles in chunk-fastest order instead of grouping the
 *    tiles of one pixel chunk on one XCD; TSM_MASK_BITS=0 (read once per process) makes the train
 *    step's data gradients take the ReLU mask of a block output from the
 *    activation itself instead of from the decision bits its forward pass keeps;
 *    TSM_SHORTCUT_BRANCH=0 (read once per process) keeps the kernels of a
 *    projection shortcut on the launch stream (they otherwise run on the library's
 *    second stream beside the residual branch, like the weight gradients, and
 *    TSM_WGRAD_OVERLAP=0 keeps everything on the launch stream).
 *  - Return value: TSM_OK or a negative tsm_status.  On error nothing has been
 *    launched (argument errors) or the stream's state is undefined
 *    (TSM_ERR_LAUNCH).  tsm_last_error() returns a host string describing the
 *    last failure on the calling thread.
 *  - Activations are the paper's five-dimensional tensor [N, T, C, H, W]
 *    (section 2, "Preliminary"), dense, in one of two memory orders:
 *      TSM_NTCHW  the order printed in the paper;
 *      TSM_NTHWC  channels innermost -- the order the MFMA kernels work in.
 *    With TSM_NTCHW the library transposes through the workspace; TSM_NTHWC is
 *    the fast path.
 *  - dtype: TSM_F32 (fp32 storage and arithmetic) or TSM_BF16 (bf16 storage,
 *    bf16 MFMA products, fp32 accumulation; all statistics, weight gradients,
 *    the loss and the optimiser state stay fp32).
 *  - Device pointers must be 16-byte aligned (TSM_ERR_ALIGN otherwise).
 *  - fold_div: 0 disables the shift (plain per-frame 2-D convolution);
 *    fold_div >= 2 moves fold = C / fold_div (integer division) channels each
 *    way; fold_div == 1 or < 0 is TSM_ERR_FOLD.
 *
 * Shift definition used throughout (the paper fixes neither the proportion nor
 * which group moves which way; this is the reading this library documents):
 *   S(x)[n,t,c]   = x[n,t+1,c]  for c <  fold           (0 when t+1 == T)
 *                 = x[n,t-1,c]  for fold <= c < 2*fold   (0 when t == 0)
 *                 = x[n,t,c]    otherwise
 *   S^T(g)[n,t,c] = g[n,t-1,c]  for c <  fold           (0 when t == 0)
 *                 = g[n,t+1,c]  for fold <= c < 2*fold   (0 when t+1 == T)
 *                 = g[n,t,c]    otherwise
 * Nothing ever crosses from clip n to clip n+1.
 */
#ifndef TSM_H
#define TSM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TSM_OK = 0,
    TSM_ERR_NULLPTR = -1,     /* a required pointer is NULL */
    TSM_ERR_SHAPE = -2,       /* non-positive or inconsistent dimension */
    TSM_ERR_FOLD = -3,        /* fold_div == 1, negative, or 2*fold > C */
    TSM_ERR_DTYPE = -4,       /* unknown dtype */
    TSM_ERR_LAYOUT = -5,      /* unknown layout */
    TSM_ERR_WORKSPACE = -6,   /* ws_bytes smaller than *_workspace_bytes() */
    TSM_ERR_ALIGN = -7,       /* device pointer not 16-byte aligned */
    TSM_ERR_LAUNCH = -8,      /* HIP reported an error; see tsm_last_error() */
    TSM_ERR_UNSUPPORTED = -9  /* valid request this build has no kernel for */
} tsm_status;

typedef enum { TSM_F32 = 0, TSM_BF16 = 1 } tsm_dtype;
typedef enum { TSM_NTCHW = 0, TSM_NTHWC = 1 } tsm_layout;

/* Host string for the last error on this thread (never NULL). */
const char* tsm_last_error(void);

/* Measurement aid, not part of the method: between tsm_profile_begin(stream) and
 * tsm_profile_end() a HIP event is recorded on `stream` after every kernel this
 * thread launches through the library; tsm_profile_end synchronises the stream
 * and writes one line per kernel class, "name launches total_ms", into the host
 * buffer `report` (NUL-terminated, truncated to report_cap).  The time booked on
 * a launch runs from the end of the previous launch to its own end. */
int tsm_profile_begin(void* stream);
int tsm_profile_end(char* report, size_t report_cap);

/* Measurement aid, not part of the method: launches a kernel of register-only
 * bf16 MFMAs (32x32x16, no memory traffic) on `stream` and writes the number
 * of floating-point operations of that launch into the host variable
 * *flops_out, so that a caller who times the launch reads the rate the matrix
 * cores sustain on this chip next to the published peak.  `iters` (1 .. 2^24)
 * MFMAs per accumulator chain; `sink` is a device float the kernel never
 * writes in practice (it keeps the arithmetic alive).  TSM_ERR_SHAPE /
 * TSM_ERR_NULLPTR on bad arguments, nothing is launched then. */
int tsm_mfma_probe(int iters, float* sink, double* flops_out, void* stream);

/* ------------------------------------------------------------------------
 * Temporal shift, stand-alone (section 2, Fig. 1: zero FLOPs, zero parameters).
 * y = S(x) / gx = S^T(gy); a pure copy, bit-exact for any 2- or 4-byte type.
 * x and y have N*T*C*H*W elements in `layout`; they must not overlap.
 * ---------------------------------------------------------------------- */
int tsm_shift_fwd(const void* x, void* y, int N, int T, int C, int H, int W,
                  int fold_div, int dtype, int layout, void* stream);
int tsm_shift_bwd(const void* gy, void* gx, int N, int T, int C, int H, int W,
                  int fold_div, int dtype, int layout, void* stream);

/* ------------------------------------------------------------------------
 * Shift-fused per-frame 2-D convolution (section 2: the network is "pure 2D
 * CNN" applied to each of the N*T frames; the shift is folded into the frame
 * index of the input load, S(x) is never materialised on the fast path).
 *   fwd:   y[f,co,oh,ow] = sum_{ci,kh,kw} w[co,ci,kh,kw] *
 *                          S(x)[f,ci,oh*stride+kh-pad,ow*stride+kw-pad]
 *   dgrad: dx = S^T( conv^T(dy, w) )
 *   wgrad: dw[co,ci,kh,kw] = sum_{f,oh,ow} dy[f,co,oh,ow] *
 *                            S(x)[f,ci,oh*stride+kh-pad,ow*stride+kw-pad]
 * x  [N,T,Cin,H,W], y/dy [N,T,Cout,Ho,Wo] in `layout`, Ho = (H+2*pad-kh)/stride+1.
 * w  [Cout,Cin,kh,kw] in `dtype`.  dw is always fp32 [Cout,Cin,kh,kw].
 * No bias (BatchNorm follows every convolution).
 * ---------------------------------------------------------------------- */
typedef struct {
    int N, T, Cin, H, W;      /* input clip tensor */
    int Cout, kh, kw;         /* filter */
    int stride, pad;
    int fold_div;             /* shift applied to the input channels */
    int dtype, layout;
} tsm_conv_desc;

/* Scratch bytes needed by the largest of the three conv calls for this desc. */
size_t tsm_conv_workspace_bytes(const tsm_conv_desc* d);

/* ch_sum / ch_sumsq: optional (both NULL or both set) fp32 [Cout] outputs that
 * receive sum_y and sum_y^2 of the stored output per channel: the BatchNorm
 * statistics epilogue.  Overwritten, not accumulated. */
int tsm_conv_fwd(const tsm_conv_desc* d, const void* x, const void* w, void* y,
                 float* ch_sum, float* ch_sumsq,
                 void* ws, size_t ws_bytes, void* stream);
int tsm_conv_dgrad(const tsm_conv_desc* d, const void* dy, const void* w, void* dx,
                   void* ws, size_t ws_bytes, void* stream);
/* tsm_conv_fwd for callers that cannot allocate device memory or supply a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error codes as
 * tsm_conv_fwd without (ws, ws_bytes): the scratch (packed weights, statistics rows, transposed copies for
 * TSM_NTCHW) is a buffer of TSM_NOALLOC_SCRATCH_BYTES that is part of the library's device image, one copy per
 * GPU, held until the process ends.  A convolution whose scratch need (tsm_conv_workspace_bytes is an upper
 * bound) exceeds that returns TSM_ERR_WORKSPACE and launches nothing.  The call allocates and frees nothing.
 * All calls on one GPU share the buffer: calls that may overlap in time on one GPU (different streams, or
 * threads) race and must be ordered by the caller; calls on one stream are ordered by the stream. */
#define TSM_NOALLOC_SCRATCH_BYTES (16u << 20)
int tsm_conv_fwd_noalloc(const tsm_conv_desc* d, const void* x, const void* w, void* y,
                         float* ch_sum, float* ch_sumsq, void* stream);
/* accumulate != 0 adds into dw instead of overwriting it (micro-batch
 * gradient accumulation, section 4.2's simulation of larger node counts). */
int tsm_conv_wgrad(const tsm_conv_desc* d, const void* x, const void* dy, float* dw,
                   int accumulate, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Residual blocks (section 3, model (3): "The TSM operator is inserted into
 * every ResBlock").  The shift sits on the residual branch in front of its
 * first convolution; the shortcut carries the unshifted input.
 *   TSM_BLOCK_BASIC       ReLU(BN(conv3x3(ReLU(BN(conv3x3(S(x)))))) + x)
 *   TSM_BLOCK_BOTTLENECK  ReLU(BN(1x1(ReLU(BN(3x3/stride(ReLU(BN(1x1(S(x))))))))) + sc(x))
 *                         sc = identity, or BN(1x1/stride conv) when has_projection
 *   TSM_BLOCK_BOTTLENECK_T3  the I3D-style comparison block (section 3, model
 *                         (2)): the first 1x1 becomes a 3x1x1 temporal
 *                         convolution (zero padding 1 in T, w1 [Cmid,Cin,3]), no shift.
 * BatchNorm is in training mode over all N*T frames: batch mean, biased batch
 * variance, eps as given.  gamma/beta and all gradients of them are fp32.
 * ---------------------------------------------------------------------- */
typedef enum { TSM_BLOCK_BASIC = 0, TSM_BLOCK_BOTTLENECK = 1, TSM_BLOCK_BOTTLENECK_T3 = 2 } tsm_block_kind;

typedef struct {
    int kind;
    int N, T, Cin, H, W;
    int Cmid, Cout;           /* BASIC: Cmid == Cout == Cin */
    int stride;               /* on the 3x3 convolution (and the projection) */
    int has_projection;
    int fold_div;
    int dtype, layout;
    float bn_eps;
} tsm_block_desc;

typedef struct {              /* device pointers; weights in desc.dtype */
    const void *w1, *w2, *w3, *wd;         /* w3: bottleneck only; wd: projection only */
    const float *g1, *b1, *g2, *b2, *g3, *b3, *gd, *bd;
} tsm_block_params;

typedef struct {              /* device pointers, all fp32, overwritten */
    float *dw1, *dw2, *dw3, *dwd;
    float *dg1, *db1, *dg2, *db2, *dg3, *db3, *dgd, *dbd;
} tsm_block_grads;

/* Bytes of the opaque, caller-owned buffer in which tsm_block_fwd keeps what
 * tsm_block_bwd needs (intermediate activations and batch statistics). */
size_t tsm_block_saved_bytes(const tsm_block_desc* d);
size_t tsm_block_workspace_bytes(const tsm_block_desc* d);

/* x [N,T,Cin,H,W] -> out [N,T,Cout,Ho,Wo]. */
int tsm_block_fwd(const tsm_block_desc* d, const void* x, const tsm_block_params* p,
                  void* out, void* saved, void* ws, size_t ws_bytes, void* stream);
/* x and out must still hold what tsm_block_fwd read and wrote; dout is the
 * gradient w.r.t. out; dx receives the gradient w.r.t. x. */
int tsm_block_bwd(const tsm_block_desc* d, const void* x, const void* out, const void* dout,
                  const void* saved, const tsm_block_params* p,
                  void* dx, const tsm_block_grads* g,
                  void* ws, size_t ws_bytes, void* stream);

/* Forward pass of one block with BatchNorm in inference mode (the mode of the paper's single-GPU throughput
 * measurement, section 3a / Table 1): every BatchNorm is the fixed map z = gamma*(y - mean)/sqrt(var + bn_eps) + beta
 * with the running statistics given here.  On the bf16 path (channels innermost) the maps, the shortcut and the
 * ReLUs ride in the convolution epilogues, and the 3x3 and the last 1x1 convolution of a bottleneck with 64 or 128
 * middle channels run as ONE kernel that keeps the tensor between them on the chip (the "hardware-friendly
 * operator" side of section 3's guideline (1): fewer bytes moved per FLOP); TSM_FUSED_TAIL=0 in the environment
 * (read at every call) keeps one kernel per convolution.  Nothing is saved for a backward pass.
 * x [N,T,Cin,H,W] -> out [N,T,Cout,Ho,Wo]; statistics fp32 [channels] per BatchNorm (m3/v3: bottlenecks only,
 * md/vd: projection only); workspace of at least tsm_block_infer_workspace_bytes(desc); errors as tsm_block_fwd. */
typedef struct {              /* device pointers, fp32: running mean and variance of each BatchNorm */
    const float *m1, *v1, *m2, *v2, *m3, *v3, *md, *vd;
} tsm_block_stats;
size_t tsm_block_infer_workspace_bytes(const tsm_block_desc* d);
int tsm_block_infer(const tsm_block_desc* d, const void* x, const tsm_block_params* p, const tsm_block_stats* st,
                    void* out, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * One training iteration of TSM-ResNet-50 on one GPU (section 3 model (3),
 * Table 1: 24.3M parameters, 33G multiply-accumulates per 8-frame clip;
 * section 4.1: SGD, weight decay not applied to BatchNorm and bias):
 * stem 7x7/2 + BN + ReLU + maxpool 3x3/2, 16 bottlenecks (3,4,6,3; stride on the
 * 3x3), global average pool, linear head per frame, mean over T, softmax
 * cross-entropy (mean over clips), full backward, SGD-momentum update
 *   g += wd*w (conv and fc weights only);  v = momentum*v + g;  w -= lr*v.
 * ---------------------------------------------------------------------- */
typedef struct {
    int N, T, size;           /* clips [N,T,3,size,size] */
    int num_classes;
    int fold_div;
    float lr, momentum, weight_decay;
    float bn_eps, bn_momentum;
    int dtype;                /* storage type of clips and activations: TSM_BF16 (MFMA path) or TSM_F32 */
} tsm_r50_desc;

/* Number of parameters (24,327,632 for 400 classes) and of parameter tensors. */
int64_t tsm_resnet50_param_count(int num_classes);
int tsm_resnet50_num_tensors(void);
/* Describes parameter tensor `index` of the flat fp32 parameter vector: name
 * (host buffer, NUL-terminated, truncated to name_cap), element offset, shape
 * (ndim <= 4; convolutions [Cout,Cin,kh,kw], head [classes,2048]), and whether
 * weight decay applies. */
int tsm_resnet50_param_info(int num_classes, int index, char* name, int name_cap,
                            int64_t* offset, int* ndim, int shape[4], int* decays);
/* Floats in the BatchNorm running-statistics buffer (mean then variance of each
 * BatchNorm, in parameter-table order). */
int64_t tsm_resnet50_bn_state_count(void);
size_t tsm_resnet50_workspace_bytes(const tsm_r50_desc* d);

/* clips   [N,T,3,size,size] of desc.dtype in the paper's order (TSM_NTCHW);
 * labels  int32 [N];
 * params, momentum   fp32 [param_count], updated in place;
 * bn_state  fp32 [bn_state_count] running mean/variance, updated in place, may be NULL;
 * grads_out fp32 [param_count] receives the raw gradients (before weight
 *           decay), may be NULL;
 * loss_out  fp32 [1]; logits_out fp32 [N,num_classes], may be NULL.
 * update != 0 applies the SGD update; 0 stops after the backward pass. */
int tsm_resnet50_step(const tsm_r50_desc* d, const void* clips, const int32_t* labels,
                      float* params, float* momentum, float* bn_state,
                      float* grads_out, float* loss_out, float* logits_out,
                      int update, void* ws, size_t ws_bytes, void* stream);

/* Inspection aid: after tsm_resnet50_step (or _accum_step) has completed on `stream`, the caller's workspace still
 * holds the forward activations the step kept for its backward pass (section 3, model (3): the tensors between
 * the layers of the stem and of the sixteen residual blocks).  This call tells where: byte `offset` from the start
 * of the workspace, `shape` = {frames N*T, rows, columns, channels} (channels innermost) and the element size
 * (desc.dtype's, 1 for the pooling positions, 4 for the fp32 vectors).  Names: "stem.y" (7x7 convolution output),
 * "stem.bn_scale" / "stem.bn_shift" (fp32 [64]: the stem's BatchNorm as the map z = scale*y + shift),
 * "stem.pool_arg" (uint8: window position kh*3+kw the 3x3/2 max-pool picked), "stem.pool" (its output), and per
 * block "res2.0." .. "res5.2.": "y1", "z1" = ReLU(BN(y1)), "y2", "z2", "y3", "yd" (projection shortcut, first
 * block of a stage) and "out".  Host-side only, no GPU work; TSM_ERR_UNSUPPORTED for an unknown name, the
 * descriptor errors of tsm_resnet50_step otherwise. */
int tsm_resnet50_workspace_tensor(const tsm_r50_desc* d, const char* name, size_t* offset, int shape[4],
                                  int* elem_bytes);

/* Gradient accumulation (the paper simulates node counts it could not run this way, section 4.2): one SGD
 * update from micro_count calls, each a forward + backward pass over its own micro-batch (its BatchNorms
 * normalise over its own N*T frames, running statistics are updated per call).  Call micro_index 0 overwrites
 * grads_accum (fp32 [param_count], caller-owned, must stay untouched between the calls) with its gradients,
 * later calls add theirs; the last call (micro_index == micro_count - 1) then applies the SGD update with
 * grads_accum / micro_count, i.e. the mean gradient over all micro-batches, and desc.lr.
 * Other arguments, workspace size and error behaviour as tsm_resnet50_step. */
int tsm_resnet50_accum_step(const tsm_r50_desc* d, const void* clips, const int32_t* labels,
                            float* params, float* momentum, float* bn_state,
                            float* grads_accum, float* loss_out, float* logits_out,
                            int micro_index, int micro_count, void* ws, size_t ws_bytes, void* stream);

/* Host-side helper (no GPU work): learning rate of the paper's recipe (section 4.1) at a fractional epoch.
 * 0.00125 per 8 samples scaled linearly with total_batch (eta = 0.00125 k for k GPUs of 8 clips); gradual
 * warm-up over the first warmup_epochs (paper: 5), rising linearly from the rate of warm_batch samples (one
 * GPU's batch, 8) to the full rate; then cosine decay reaching 0 at total_epochs (paper: 100).
 * Returns -1 (and sets tsm_last_error) for invalid arguments. */
double tsm_lr_schedule(double epoch, int total_batch, int warm_batch, double warmup_epochs, double total_epochs);

/* Forward pass only, BatchNorm in inference mode (the way the paper measures single-GPU
 * throughput of the models: section 3a, Table 1, videos per second at batch 16).
 * Every BatchNorm uses the running statistics in bn_state (layout as above) instead of batch statistics:
 * z = gamma*(y - mean)/sqrt(var + bn_eps) + beta.  On the bf16 path this affine map, the shortcut and the
 * ReLU are applied in the epilogue of the convolution that produces y.
 * Uses of desc: N, T, size, num_classes, fold_div, bn_eps, dtype (the optimiser fields are ignored).
 * clips as for tsm_resnet50_step; params fp32 [param_count] (read only); bn_state fp32 [bn_state_count]
 * (read only, required); logits_out fp32 [N,num_classes]: mean over the T per-frame predictions.
 * All pointers are device pointers; the call is asynchronous on `stream`; ws is caller-owned scratch of at
 * least tsm_resnet50_infer_workspace_bytes(desc) bytes (0 is returned for an invalid descriptor). */
size_t tsm_resnet50_infer_workspace_bytes(const tsm_r50_desc* d);
int tsm_resnet50_infer(const tsm_r50_desc* d, const void* clips, const float* params,
                       const float* bn_state, float* logits_out,
                       void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TSM_H */
