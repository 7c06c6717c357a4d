// C-ABI entry points for the shift-fused convolutions and the residual blocks,
// and the internal block driver the TSM-ResNet-50 step reuses.
#include <algorithm>
#include <mutex>
#include "internal.h"
#include "block.h"

namespace tsm {

#define RUN(expr)                          \
    do {                                   \
        if (!dry) TSM_TRY(expr);           \
    } while (0)

// ---- descriptor checks -----------------------------------------------------------
static int check_common(int dtype, int layout, const char* who) {
    if (dtype != TSM_F32 && dtype != TSM_BF16) return fail(TSM_ERR_DTYPE, "%s: unknown dtype %d", who, dtype);
    if (layout != TSM_NTCHW && layout != TSM_NTHWC) return fail(TSM_ERR_LAYOUT, "%s: unknown layout %d", who, layout);
    return TSM_OK;
}

static int make_convp(const tsm_conv_desc* d, ConvP* p, const char* who) {
    if (!d) return fail(TSM_ERR_NULLPTR, "%s: null descriptor", who);
    TSM_TRY(check_common(d->dtype, d->layout, who));
    if (d->N <= 0 || d->T <= 0 || d->Cin <= 0 || d->H <= 0 || d->W <= 0 || d->Cout <= 0 || d->kh <= 0 || d->kw <= 0 ||
        d->stride <= 0 || d->pad < 0)
        return fail(TSM_ERR_SHAPE, "%s: non-positive dimension", who);
    if (d->H + 2 * d->pad < d->kh || d->W + 2 * d->pad < d->kw) return fail(TSM_ERR_SHAPE, "%s: filter larger than padded frame", who);
    if ((long)d->N * d->T > 0x7fffffffL / 4) return fail(TSM_ERR_SHAPE, "%s: too many frames", who);
    int fold = 0;
    if (fold_of(d->Cin, d->fold_div, &fold) != TSM_OK) return fail(TSM_ERR_FOLD, "%s: invalid fold_div %d for Cin=%d", who, d->fold_div, d->Cin);
    p->F = d->N * d->T; p->T = d->T; p->H = d->H; p->W = d->W; p->Cin = d->Cin;
    p->Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1;
    p->Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    p->Cout = d->Cout; p->KT = 1; p->KH = d->kh; p->KW = d->kw; p->stride = d->stride; p->pad = d->pad;
    p->fold = fold;
    return TSM_OK;
}

static inline bool use_mfma(const ConvP& p, int dtype) { return dtype == TSM_BF16 && mfma_conv_supported(p); }

// ---- internal conv runners (channels-innermost) -----------------------------------------
// Rows of the statistics partial buffer run_conv_fwd fills for this convolution.
int conv_stats_blocks(const ConvP& p, int dtype) {
    return use_mfma(p, dtype) ? conv_mfma_fwd_blocks(p) : red_blocks(p.rows_out(), p.Cout, dtype);
}

// stats_partial: fp32 [conv_stats_blocks(p, dtype)][2*Cout] or null.
int run_conv_fwd(const ConvP& p, int dtype, const void* x, const void* w, const bf16_t* wp, void* y,
                 float* stats_partial, Arena& ws, bool dry, hipStream_t s) {
    if (use_mfma(p, dtype)) {
        if (!wp) {
            bf16_t* pk = ws.take_n<bf16_t>((size_t)p.Cout * p.K());
            RUN(pack_weights_fwd(dtype, w, pk, p.Cout, p.Cin, p.taps(), p.Cin, s));
            wp = pk;
        }
        RUN(conv_mfma_fwd(p, (const bf16_t*)x, wp, (bf16_t*)y, stats_partial, nullptr, s));
    } else {
        RUN(conv_direct_fwd(p, dtype, x, w, y, s));
        if (stats_partial) RUN(channel_stats(dtype, y, p.rows_out(), p.Cout, stats_partial, s));
    }
    return TSM_OK;
}

int conv_dgrad_fuse_blocks(const ConvP& p, int dtype) { return use_mfma(p, dtype) ? conv_mfma_dgrad_blocks(p) : 0; }

int run_conv_dgrad(const ConvP& p, int dtype, const void* dy, const void* w, const bf16_t* wd, void* dx,
                   const void* addend, const DgradFuse* fuse, Arena& ws, bool dry, hipStream_t s, int addend_stride) {
    if (fuse && !use_mfma(p, dtype)) return fail(TSM_ERR_UNSUPPORTED, "dgrad: no fused path for this layer");
    if (addend_stride != 1 && !use_mfma(p, dtype)) return fail(TSM_ERR_UNSUPPORTED, "dgrad: no compact addend for this layer");
    if (use_mfma(p, dtype)) {
        if (!wd) {
            bf16_t* pk = ws.take_n<bf16_t>((size_t)p.Cout * p.K());
            RUN(pack_weights_dgrad(dtype, w, pk, p.Cout, p.Cin, p.KT, p.KH, p.KW, s));
            wd = pk;
        }
        RUN(conv_mfma_dgrad(p, (const bf16_t*)dy, wd, (bf16_t*)dx, (const bf16_t*)addend, fuse, s, addend_stride));
    } else {
        RUN(conv_direct_dgrad(p, dtype, dy, w, dx, addend, s));
    }
    return TSM_OK;
}

int run_conv_wgrad(const ConvP& p, int dtype, const void* x, const void* dy, float* dw, float* dwp_zeroed, int accumulate,
                   Arena& ws, bool dry, hipStream_t s) {
    // all kernels add with atomics; "accumulate" skips the zero fill of dw
    const size_t n = (size_t)p.Cout * p.K();
    if (use_mfma(p, dtype) && p.taps() > 1 && dwp_zeroed) {
        // the caller owns a zeroed packed buffer and permutes it into dw later (one fill / one permutation per step)
        RUN(conv_mfma_wgrad(p, (const bf16_t*)x, (const bf16_t*)dy, dwp_zeroed, p.Cin, true, s));
        return TSM_OK;
    }
    if (use_mfma(p, dtype) && p.taps() > 1) {
        // several taps: accumulate in the packed order (contiguous atomics), then permute into dw
        float* dwp = ws.take_n<float>(n);
        RUN(fill_zero(dwp, n * sizeof(float), s));
        RUN(conv_mfma_wgrad(p, (const bf16_t*)x, (const bf16_t*)dy, dwp, p.Cin, true, s));
        RUN(unpack_wgrad(dwp, dw, p.Cout, p.Cin, p.taps(), p.Cin, accumulate, s));
        return TSM_OK;
    }
    if (!accumulate) RUN(fill_zero(dw, n * sizeof(float), s));
    if (use_mfma(p, dtype))
        RUN(conv_mfma_wgrad(p, (const bf16_t*)x, (const bf16_t*)dy, dw, p.Cin, false, s));
    else
        RUN(conv_direct_wgrad(p, dtype, x, dy, dw, s));
    return TSM_OK;
}

// ---- conv entry points -------------------------------------------------------------------
enum { CONV_FWD = 0, CONV_DGRAD = 1, CONV_WGRAD = 2 };

static int conv_entry(int which, const tsm_conv_desc* d, const void* a0, const void* a1, void* out, float* ch_sum,
                      float* ch_sumsq, int accumulate, void* wsp, size_t ws_bytes, bool dry, hipStream_t s,
                      size_t* need) {
    const char* who = which == CONV_FWD ? "tsm_conv_fwd" : which == CONV_DGRAD ? "tsm_conv_dgrad" : "tsm_conv_wgrad";
    ConvP p;
    TSM_TRY(make_convp(d, &p, who));
    if (!dry) {
        if (!a0 || !a1 || !out) return fail(TSM_ERR_NULLPTR, "%s: null tensor pointer", who);
        if ((ch_sum == nullptr) != (ch_sumsq == nullptr)) return fail(TSM_ERR_NULLPTR, "%s: ch_sum and ch_sumsq must both be set or both be NULL", who);
        if (!aligned16(a0) || !aligned16(a1) || !aligned16(out) || !aligned16(wsp))
            return fail(TSM_ERR_ALIGN, "%s: pointers must be 16-byte aligned", who);
        if (ws_bytes > 0 && !wsp) return fail(TSM_ERR_NULLPTR, "%s: null workspace", who);
    }
    Arena ws(dry ? nullptr : wsp, dry ? (size_t)-1 : ws_bytes);
    if (!dry) {  // size check first, with a dry pass of the same plan
        size_t req = 0;
        TSM_TRY(conv_entry(which, d, a0, a1, out, ch_sum, ch_sumsq, accumulate, nullptr, 0, true, s, &req));
        if (req > ws_bytes) return fail(TSM_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu", who, ws_bytes, req);
    }
    const int es = (int)dtype_size(d->dtype);
    const size_t xin = (size_t)p.rows_in() * p.Cin * es, yout = (size_t)p.rows_out() * p.Cout * es;
    const bool tr = d->layout == TSM_NTCHW;
    if (which == CONV_FWD) {
        const void* x = a0;
        void* y = out;
        if (tr) {
            void* xt = ws.take(xin);
            y = ws.take(yout);
            RUN(transpose_frames(a0, xt, p.F, p.Cin, p.H * p.W, es, s));
            x = xt;
        }
        const int nb = conv_stats_blocks(p, d->dtype);
        float* part = (ch_sum || dry) ? ws.take_n<float>((size_t)nb * 2 * p.Cout) : nullptr;
        TSM_TRY(run_conv_fwd(p, d->dtype, x, a1, nullptr, y, ch_sum ? part : nullptr, ws, dry, s));
        if (ch_sum) RUN(stats_to_float(part, nb, p.Cout, ch_sum, ch_sumsq, s));
        if (tr) RUN(transpose_frames(y, out, p.F, p.Ho * p.Wo, p.Cout, es, s));
    } else if (which == CONV_DGRAD) {
        const void* dy = a0;
        void* dx = out;
        if (tr) {
            void* dyt = ws.take(yout);
            dx = ws.take(xin);
            RUN(transpose_frames(a0, dyt, p.F, p.Cout, p.Ho * p.Wo, es, s));
            dy = dyt;
        }
        TSM_TRY(run_conv_dgrad(p, d->dtype, dy, a1, nullptr, dx, nullptr, nullptr, ws, dry, s));
        if (tr) RUN(transpose_frames(dx, out, p.F, p.H * p.W, p.Cin, es, s));
    } else {
        const void *x = a0, *dy = a1;
        if (tr) {
            void* xt = ws.take(xin);
            void* dyt = ws.take(yout);
            RUN(transpose_frames(a0, xt, p.F, p.Cin, p.H * p.W, es, s));
            RUN(transpose_frames(a1, dyt, p.F, p.Cout, p.Ho * p.Wo, es, s));
            x = xt;
            dy = dyt;
        }
        TSM_TRY(run_conv_wgrad(p, d->dtype, x, dy, (float*)out, nullptr, accumulate, ws, dry, s));
    }
    if (need) *need = ws.used;
    return TSM_OK;
}

// ---- residual blocks ---------------------------------------------------------------------
static size_t bnvec_take(Arena& a, int C, BnVec* v) {
    v->mean = a.take_n<float>(C);
    v->rstd = a.take_n<float>(C);
    v->scale = a.take_n<float>(C);
    v->shift = a.take_n<float>(C);
    return 0;
}

// Lays the saved buffer out (same order in fwd and bwd).
void block_saved_layout(BlockPlan& b, Arena& sv, bool keep_x_copy) {
    const int es = (int)dtype_size(b.dtype);
    if (keep_x_copy) {
        b.x_copy = sv.take((size_t)b.st[0].p.rows_in() * b.st[0].p.Cin * es);
        b.out_copy = sv.take((size_t)b.st[b.nst - 1].p.rows_out() * b.st[b.nst - 1].p.Cout * es);
    }
    for (int i = 0; i < b.nst; ++i) {
        const ConvP& p = b.st[i].p;
        b.y[i] = sv.take((size_t)p.rows_out() * p.Cout * es);
        if (i + 1 < b.nst) b.z[i] = sv.take((size_t)p.rows_out() * p.Cout * es);
        bnvec_take(sv, p.Cout, &b.bn[i]);
    }
    if (b.proj) {
        const ConvP& p = b.ds.p;
        b.yd = sv.take((size_t)p.rows_out() * p.Cout * es);
        bnvec_take(sv, p.Cout, &b.bnd);
    }
}

// ---- weight gradients beside the data-gradient chain -----------------------------------------------------
// A weight gradient only feeds the optimiser, so inside one block's backward pass it runs on a second stream
// (default priority) while the main stream goes on with the data gradients: fork = the side stream waits for an
// event recorded on the main stream after the kernel that produced the weight gradient's operand; join = the main
// stream waits, at the end of the block, for an event recorded behind the last weight gradient.  Nothing the
// weight gradients read is rewritten inside the block, and the join comes before the block's scratch is reused.
// Per host thread and device; TSM_WGRAD_OVERLAP=0, per-launch profiling or a failed stream creation keep
// everything on the caller's stream.  The first call on a device creates the stream and events (do not make that
// call under stream capture; later calls capture as a fork/join pattern).
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    hipEvent_t lag[2] = {nullptr, nullptr};   // joins that the launch stream takes one block late (see block_bwd_impl)
    hipEvent_t branch = nullptr;              // end of a projection shortcut's work on the side stream
    bool pending[2] = {false, false};
    int state = 0;   // 0 untried, 1 ready, -1 unavailable
};

static SideStream* side_stream() {
    static int enabled = -1;
    if (enabled < 0) {
        const char* e = getenv("TSM_WGRAD_OVERLAP");
        enabled = (e && e[0] == '0') ? 0 : 1;
    }
    if (!enabled || profiling_active()) return nullptr;
    static thread_local SideStream side[16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
    SideStream& ss = side[dev];
    if (ss.state == 0) {
        ss.state = -1;
        if (hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ss.join, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ss.lag[0], hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ss.lag[1], hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ss.branch, hipEventDisableTiming) == hipSuccess)
            ss.state = 1;
        else
            (void)hipGetLastError();
    }
    return ss.state == 1 ? &ss : nullptr;
}

// Runs one weight gradient on the side stream behind everything enqueued on `s` so far (or on `s` itself).
static int wgrad_beside(SideStream* ss, bool* forked, const ConvP& p, int dtype, const void* x, const void* dy, float* dw,
                        float* dwp, int accumulate, Arena& ws, bool dry, hipStream_t s) {
    if (!ss || dry) return run_conv_wgrad(p, dtype, x, dy, dw, dwp, accumulate, ws, dry, s);
    if (hipEventRecord(ss->fork, s) != hipSuccess || hipStreamWaitEvent(ss->stream, ss->fork, 0) != hipSuccess)
        return fail(TSM_ERR_LAUNCH, "block backward: cannot fork the weight-gradient stream");
    *forked = true;
    return run_conv_wgrad(p, dtype, x, dy, dw, dwp, accumulate, ws, dry, ss->stream);
}

// A branch of independent work for a caller inside the library: the side stream, forked behind everything enqueued on
// `s` so far (or `s` itself where there is no side stream); side_branch_end joins it (a no-op for `s` itself).
hipStream_t side_branch_begin(hipStream_t s) {
    SideStream* const ss = side_stream();
    if (!ss) return s;
    if (hipEventRecord(ss->fork, s) != hipSuccess || hipStreamWaitEvent(ss->stream, ss->fork, 0) != hipSuccess) {
        (void)hipGetLastError();
        return s;
    }
    return ss->stream;
}

int side_branch_end(hipStream_t s, hipStream_t branch) {
    if (branch == s) return TSM_OK;
    SideStream* const ss = side_stream();
    if (!ss || hipEventRecord(ss->join, ss->stream) != hipSuccess || hipStreamWaitEvent(s, ss->join, 0) != hipSuccess)
        return fail(TSM_ERR_LAUNCH, "cannot join the side stream");
    return TSM_OK;
}

// TSM_SHORTCUT_BRANCH=0 (read once per process) keeps a projection shortcut's kernels on the launch stream.
static bool shortcut_branch_enabled() {
    static int enabled = -1;
    if (enabled < 0) {
        const char* e = getenv("TSM_SHORTCUT_BRANCH");
        enabled = (e && e[0] == '0') ? 0 : 1;
    }
    return enabled != 0;
}

static int wgrad_join(SideStream* ss, bool forked, hipStream_t s) {
    if (!ss || !forked) return TSM_OK;
    if (hipEventRecord(ss->join, ss->stream) != hipSuccess || hipStreamWaitEvent(s, ss->join, 0) != hipSuccess)
        return fail(TSM_ERR_LAUNCH, "block backward: cannot join the weight-gradient stream");
    return TSM_OK;
}

// The projection shortcut (convolution + BatchNorm statistics) depends on the block input only: it runs on the side
// stream beside the first convolution, which reads the same tensor, and is joined in front of the block's tail.
static int block_fwd_stages(BlockPlan& b, const void* x, Arena& ws, bool dry, hipStream_t s) {
    const void* cur = x;
    for (int i = 0; i < b.nst; ++i) {
        StageDef& st = b.st[i];
        const int nb = conv_stats_blocks(st.p, b.dtype);
        float* part = ws.take_n<float>((size_t)nb * 2 * st.p.Cout);
        TSM_TRY(run_conv_fwd(st.p, b.dtype, cur, st.w, st.wp, b.y[i], part, ws, dry, s));
        RUN(bn_finalize(part, nb, st.p.rows_out(), st.p.Cout, st.g, st.b, b.eps, b.bn[i], st.run_mean, st.run_var,
                        b.bn_momentum, s));
        if (i + 1 < b.nst) {
            RUN(bn_relu_apply(b.dtype, b.y[i], st.p.rows_out(), st.p.Cout, b.bn[i].scale, b.bn[i].shift, b.z[i], s));
            cur = b.z[i];
        }
    }
    return TSM_OK;
}

static int block_fwd_shortcut(BlockPlan& b, const void* x, Arena& ws, bool dry, hipStream_t s) {
    StageDef& st = b.ds;
    const int nb = conv_stats_blocks(st.p, b.dtype);
    float* part = ws.take_n<float>((size_t)nb * 2 * st.p.Cout);
    TSM_TRY(run_conv_fwd(st.p, b.dtype, x, st.w, st.wp, b.yd, part, ws, dry, s));
    RUN(bn_finalize(part, nb, st.p.rows_out(), st.p.Cout, st.g, st.b, b.eps, b.bnd, st.run_mean, st.run_var,
                    b.bn_momentum, s));
    return TSM_OK;
}

int block_fwd_impl(BlockPlan& b, const void* x, void* out, Arena& ws, bool dry, hipStream_t s) {
    SideStream* const ss = (dry || !b.proj || !shortcut_branch_enabled()) ? nullptr : side_stream();
    bool forked = false;
    int rc = TSM_OK;
    if (b.proj) {
        hipStream_t sd = s;
        if (ss) {
            if (hipEventRecord(ss->fork, s) != hipSuccess || hipStreamWaitEvent(ss->stream, ss->fork, 0) != hipSuccess)
                return fail(TSM_ERR_LAUNCH, "block forward: cannot fork the side stream");
            forked = true;
            sd = ss->stream;
        }
        rc = block_fwd_shortcut(b, x, ws, dry, sd);
    }
    if (rc == TSM_OK) rc = block_fwd_stages(b, x, ws, dry, s);
    const int rj = wgrad_join(ss, forked, s);      // on every path: a caller's stream capture must not keep an open branch
    if (rc != TSM_OK) return rc;
    if (rj != TSM_OK) return rj;
    const int L = b.nst - 1;
    const ConvP& pl = b.st[L].p;
    RUN(block_tail_fwd(b.dtype, b.y[L], pl.rows_out(), pl.Cout, b.bn[L].scale, b.bn[L].shift, b.proj ? b.yd : x,
                       b.proj ? b.bnd.scale : nullptr, b.proj ? b.bnd.shift : nullptr, out, s, b.out_bits));
    return TSM_OK;
}

// ---- forward only, BatchNorm with known statistics (inference) -------------------------------------------------
// out = act(scale*conv(x) + shift + res): in the convolution's epilogue where its kernel can, else the raw
// convolution into ytmp and an elementwise pass.
static int conv_affine_fwd(const StageDef& sd, int dtype, const bf16_t* wp, const void* x, const float* sc, const float* sh,
                           const void* res, int relu, void* out, void* ytmp, Arena& ws, bool dry, hipStream_t s) {
    if (use_mfma(sd.p, dtype) && wp && conv_mfma_fwd_can_fuse(sd.p)) {
        const FwdEpilogue ep = {sc, sh, (const bf16_t*)res, relu};
        RUN(conv_mfma_fwd(sd.p, (const bf16_t*)x, wp, (bf16_t*)out, nullptr, &ep, s));
        return TSM_OK;
    }
    if (!relu) return fail(TSM_ERR_UNSUPPORTED, "inference: no unfused path for an affine map without ReLU");
    TSM_TRY(run_conv_fwd(sd.p, dtype, x, sd.w, wp, ytmp, nullptr, ws, dry, s));
    if (res)
        RUN(block_tail_fwd(dtype, ytmp, sd.p.rows_out(), sd.p.Cout, sc, sh, res, nullptr, nullptr, out, s));
    else
        RUN(bn_relu_apply(dtype, ytmp, sd.p.rows_out(), sd.p.Cout, sc, sh, out, s));
    return TSM_OK;
}

int block_infer_impl(BlockPlan& b, const InferParams& ip, const void* x, void* out, void* mid0, void* mid1, void* ytmp,
                     void* scbuf, Arena& ws, bool dry, hipStream_t s) {
    const int L = b.nst - 1;
    const bool bf = b.dtype == TSM_BF16;
    // the projection shortcut first: BatchNorm(conv(x)) by the affine epilogue where the kernel has one
    const bool proj_fused = b.proj && use_mfma(b.ds.p, b.dtype) && ip.wp[3] && conv_mfma_fwd_can_fuse(b.ds.p);
    // the last two convolutions of a bottleneck as one kernel (the tensor between them stays on the chip)
    const bool tail = bf && b.nst == 3 && ip.wp[1] && ip.wp[2] && (!b.proj || proj_fused) && use_mfma(b.st[1].p, b.dtype) &&
                      use_mfma(b.st[2].p, b.dtype) && conv_mfma_fused_tail_supported(b.st[1].p, b.st[2].p);
    const void* cur = x;
    void* mids[2] = {mid0, mid1};
    const int plain_stages = tail ? 1 : L;
    for (int i = 0; i < plain_stages; ++i) {
        TSM_TRY(conv_affine_fwd(b.st[i], b.dtype, ip.wp[i], cur, ip.sc[i], ip.sh[i], nullptr, 1, mids[i & 1], ytmp, ws, dry, s));
        cur = mids[i & 1];
    }
    const void* res = x;
    if (b.proj) {
        if (proj_fused) {
            const FwdEpilogue ep = {ip.sc[3], ip.sh[3], nullptr, 0};
            RUN(conv_mfma_fwd(b.ds.p, (const bf16_t*)x, ip.wp[3], (bf16_t*)scbuf, nullptr, &ep, s));
            res = scbuf;
        } else {
            // unfused: both raw convolution outputs, then one pass relu(bn(y) + bn_d(yd))
            TSM_TRY(run_conv_fwd(b.ds.p, b.dtype, x, b.ds.w, ip.wp[3], scbuf, nullptr, ws, dry, s));
            TSM_TRY(run_conv_fwd(b.st[L].p, b.dtype, cur, b.st[L].w, ip.wp[L], ytmp, nullptr, ws, dry, s));
            RUN(block_tail_fwd(b.dtype, ytmp, b.st[L].p.rows_out(), b.st[L].p.Cout, ip.sc[L], ip.sh[L], scbuf, ip.sc[3],
                               ip.sh[3], out, s));
            return TSM_OK;
        }
    }
    if (tail) {
        RUN(conv_mfma_fused_tail(b.st[1].p, b.st[2].p, (const bf16_t*)cur, ip.wp[1], ip.wp[2], ip.sc[1], ip.sh[1], ip.sc[2],
                                 ip.sh[2], (const bf16_t*)res, (bf16_t*)out, s));
        return TSM_OK;
    }
    return conv_affine_fwd(b.st[L], b.dtype, ip.wp[L], cur, ip.sc[L], ip.sh[L], res, 1, out, ytmp, ws, dry, s);
}

static void bind_params(BlockPlan& b, const tsm_block_params* p, const tsm_block_grads* g);
static int check_block_ptrs(const BlockPlan& b, bool bwd, const char* who);

static int block_infer_entry(const tsm_block_desc* d, const void* x, const tsm_block_params* prm, const tsm_block_stats* st,
                             void* out, void* wsp, size_t ws_bytes, bool dry, hipStream_t s, size_t* need) {
    const char* who = "tsm_block_infer";
    BlockPlan b;
    TSM_TRY(make_block_plan(d, &b, who));
    const bool tr = d->layout == TSM_NTCHW;
    if (!dry) {
        if (!prm || !st) return fail(TSM_ERR_NULLPTR, "%s: null params or statistics", who);
        bind_params(b, prm, nullptr);
        TSM_TRY(check_block_ptrs(b, false, who));
        const float* mv[8] = {st->m1, st->v1, st->m2, st->v2, st->m3, st->v3, st->md, st->vd};
        for (int i = 0; i < b.nst; ++i)
            if (!mv[2 * i] || !mv[2 * i + 1]) return fail(TSM_ERR_NULLPTR, "%s: null running statistics (stage %d)", who, i + 1);
        if (b.proj && (!st->md || !st->vd)) return fail(TSM_ERR_NULLPTR, "%s: null running statistics (projection)", who);
        if (!x || !out) return fail(TSM_ERR_NULLPTR, "%s: null tensor pointer", who);
        if (!aligned16(x) || !aligned16(out) || !aligned16(wsp)) return fail(TSM_ERR_ALIGN, "%s: pointers must be 16-byte aligned", who);
        size_t req = 0;
        TSM_TRY(block_infer_entry(d, x, prm, st, out, nullptr, 0, true, s, &req));
        if (req > ws_bytes) return fail(TSM_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu", who, ws_bytes, req);
        if (req > 0 && !wsp) return fail(TSM_ERR_NULLPTR, "%s: null workspace", who);
    }
    Arena ws(dry ? nullptr : wsp, dry ? (size_t)-1 : ws_bytes);
    const int es = (int)dtype_size(d->dtype);
    const ConvP& p0 = b.st[0].p;
    const ConvP& pl = b.st[b.nst - 1].p;
    const size_t out_bytes = (size_t)pl.rows_out() * pl.Cout * es;
    size_t mid_bytes = 0;
    for (int i = 0; i + 1 < b.nst; ++i) mid_bytes = std::max(mid_bytes, (size_t)b.st[i].p.rows_out() * b.st[i].p.Cout * es);
    void* mid0 = ws.take(mid_bytes);
    void* mid1 = ws.take(mid_bytes);
    void* ytmp = ws.take(out_bytes);
    void* scbuf = ws.take(out_bytes);
    InferParams ip{};
    const StageDef* sds[4] = {&b.st[0], &b.st[1], b.nst == 3 ? &b.st[2] : nullptr, b.proj ? &b.ds : nullptr};
    const float* mean[4] = {dry ? nullptr : st->m1, dry ? nullptr : st->m2, dry ? nullptr : st->m3, dry ? nullptr : st->md};
    const float* var[4] = {dry ? nullptr : st->v1, dry ? nullptr : st->v2, dry ? nullptr : st->v3, dry ? nullptr : st->vd};
    for (int i = 0; i < 4; ++i) {
        if (!sds[i]) continue;
        const ConvP& p = sds[i]->p;
        float* sc = ws.take_n<float>(p.Cout);
        float* sh = ws.take_n<float>(p.Cout);
        RUN(bn_eval_vec(sds[i]->g, sds[i]->b, mean[i], var[i], d->bn_eps, p.Cout, sc, sh, s));
        ip.sc[i] = sc;
        ip.sh[i] = sh;
        if (use_mfma(p, d->dtype)) {
            bf16_t* pk = ws.take_n<bf16_t>((size_t)p.Cout * p.K());
            RUN(pack_weights_fwd(d->dtype, sds[i]->w, pk, p.Cout, p.Cin, p.taps(), p.Cin, s));
            ip.wp[i] = pk;
        }
    }
    const void* xi = x;
    void* oi = out;
    if (tr) {
        void* xt = ws.take((size_t)p0.rows_in() * p0.Cin * es);
        oi = ws.take(out_bytes);
        RUN(transpose_frames(x, xt, p0.F, p0.Cin, p0.H * p0.W, es, s));
        xi = xt;
    }
    TSM_TRY(block_infer_impl(b, ip, xi, oi, mid0, mid1, ytmp, scbuf, ws, dry, s));
    if (tr) RUN(transpose_frames(oi, out, pl.F, pl.Ho * pl.Wo, pl.Cout, es, s));
    if (need) *need = ws.used;
    return TSM_OK;
}

// The body of block_bwd_impl; `forked` tells the caller whether the side stream has work of this block, so that it
// is joined on every path out, errors included (a caller's stream capture must not be left with an open branch).
static int block_bwd_body(BlockPlan& b, const void* x, const void* out, const void* dout, void* dx, Arena& ws, bool dry,
                          hipStream_t s, SideStream* ss, bool& forked);

// Takes the joins that block_bwd_impl left open in its late-join mode.
int block_bwd_flush(hipStream_t s) {
    SideStream* const ss = side_stream();
    int rc = TSM_OK;
    if (!ss) return rc;
    for (int k = 0; k < 2; ++k) {
        if (!ss->pending[k]) continue;
        ss->pending[k] = false;
        if (hipStreamWaitEvent(s, ss->lag[k], 0) != hipSuccess) rc = fail(TSM_ERR_LAUNCH, "block backward: cannot join the weight-gradient stream");
    }
    return rc;
}

// lag_slot < 0: the launch stream joins the weight-gradient stream at the end of the block.  lag_slot 0 / 1 (a chain of
// blocks whose scratch alternates between two regions, slot = region): the join of this block is left open and the one
// the previous call left open -- the other slot's -- is taken instead, so the weight gradients of a block may run on
// beside the next block's kernels and are complete before the block after that reuses their scratch region.  The
// caller ends the chain with block_bwd_flush, on every path.
int block_bwd_impl(BlockPlan& b, const void* x, const void* out, const void* dout, void* dx, Arena& ws, bool dry,
                   hipStream_t s, int lag_slot) {
    SideStream* const ss = dry ? nullptr : side_stream();
    bool forked = false;
    const int rc = block_bwd_body(b, x, out, dout, dx, ws, dry, s, ss, forked);
    if (lag_slot >= 0 && ss && rc == TSM_OK) {
        const int k = lag_slot & 1;
        if (ss->pending[k]) return fail(TSM_ERR_LAUNCH, "block backward: the scratch region of this slot is still in use");
        if (forked) {
            if (hipEventRecord(ss->lag[k], ss->stream) != hipSuccess) {
                (void)wgrad_join(ss, true, s);
                return fail(TSM_ERR_LAUNCH, "block backward: cannot record the weight-gradient stream's join");
            }
            ss->pending[k] = true;
        }
        if (ss->pending[k ^ 1]) {
            ss->pending[k ^ 1] = false;
            if (hipStreamWaitEvent(s, ss->lag[k ^ 1], 0) != hipSuccess)
                return fail(TSM_ERR_LAUNCH, "block backward: cannot join the weight-gradient stream");
        }
        return TSM_OK;
    }
    const int rj = wgrad_join(ss, forked, s);
    return rc != TSM_OK ? rc : rj;
}

static int block_bwd_body(BlockPlan& b, const void* x, const void* out, const void* dout, void* dx, Arena& ws, bool dry,
                          hipStream_t s, SideStream* ss, bool& forked) {
    const int es = (int)dtype_size(b.dtype);
    const int L = b.nst - 1;
    const ConvP& pl = b.st[L].p;
    const size_t out_bytes = (size_t)pl.rows_out() * pl.Cout * es;
    void* dzL = ws.take(out_bytes);
    void* dyL = ws.take(out_bytes);
    const bool chained = b.dout_part != nullptr;   // dout is dz already, its sums are in dout_part
    if (chained && b.proj) return fail(TSM_ERR_UNSUPPORTED, "block backward: a chained gradient needs an identity shortcut");
    const int nbL = chained ? b.dout_nb : red_blocks(pl.rows_out(), pl.Cout, b.dtype);
    float* partL = ws.take_n<float>((size_t)nbL * 2 * pl.Cout);
    float* partd = ws.take_n<float>((size_t)nbL * 2 * pl.Cout);
    float* coefL = ws.take_n<float>(3 * (size_t)pl.Cout);
    const int acc_flag = b.grads_prezeroed ? 1 : 0;
    if (chained) {
        dzL = const_cast<void*>(dout);
        partL = const_cast<float*>(b.dout_part);
    } else if (b.dout_masked) {
        // dout is dz already (the producing data gradient applied the mask): only the sums are taken
        dzL = const_cast<void*>(dout);
        RUN(relu_bn_bwd_reduce(b.dtype, dout, nullptr, b.y[L], pl.rows_out(), pl.Cout, b.bn[L].mean, b.bn[L].rstd, nullptr, partL,
                               b.proj ? b.yd : nullptr, b.proj ? b.bnd.mean : nullptr, b.proj ? b.bnd.rstd : nullptr,
                               b.proj ? partd : nullptr, s));
    } else {
        RUN(relu_bn_bwd_reduce(b.dtype, dout, out, b.y[L], pl.rows_out(), pl.Cout, b.bn[L].mean, b.bn[L].rstd, dzL, partL,
                               b.proj ? b.yd : nullptr, b.proj ? b.bnd.mean : nullptr, b.proj ? b.bnd.rstd : nullptr,
                               b.proj ? partd : nullptr, s));
    }
    RUN(bn_bwd_coeffs(partL, nbL, pl.rows_out(), pl.Cout, b.bn[L].mean, b.bn[L].rstd, b.st[L].g, coefL, b.st[L].dg,
                      b.st[L].db, s));
    // a projection shortcut's BatchNorm takes the same upstream gradient: both are applied from one read of it
    void* dyd = nullptr;
    if (b.proj) {
        dyd = ws.take(out_bytes);
        float* coefd = ws.take_n<float>(3 * (size_t)pl.Cout);
        RUN(bn_bwd_coeffs(partd, nbL, pl.rows_out(), pl.Cout, b.bnd.mean, b.bnd.rstd, b.ds.g, coefd, b.ds.dg, b.ds.db, s));
        RUN(bn_bwd_apply2(b.dtype, dzL, b.y[L], coefL, dyL, b.yd, coefd, dyd, pl.rows_out(), pl.Cout, s));
    } else {
        RUN(bn_bwd_apply(b.dtype, dzL, b.y[L], pl.rows_out(), pl.Cout, coefL, dyL, s));
    }
    // The projection shortcut's data gradient depends on dyd only and is needed by the block's last data gradient only:
    // it runs on the side stream, behind the last stage's weight gradient, beside the chain of the residual branch.
    const void* addend = dzL;
    int addend_stride = 1;
    bool branch_open = false;
    SideStream* const ss_all = ss;
    auto shortcut_dgrad = [&]() -> int {
        StageDef& st = b.ds;
        void* dsc = ws.take((size_t)st.p.rows_in() * st.p.Cin * es);
        hipStream_t sd = s;
        SideStream* const ss = shortcut_branch_enabled() ? ss_all : nullptr;
        if (ss) {
            if (hipEventRecord(ss->fork, s) != hipSuccess || hipStreamWaitEvent(ss->stream, ss->fork, 0) != hipSuccess)
                return fail(TSM_ERR_LAUNCH, "block backward: cannot fork the side stream");
            forked = true;
            sd = ss->stream;
        }
        // A 1x1 projection with stride 2 sends gradient only to the input pixels with even row and column: its data
        // gradient is the 1x1 stride-1 data gradient on the output grid, kept in that compact form and added at the
        // even pixels by the kernel that produces dx (three quarters of the tensor are neither written nor read)
        if (st.p.stride == 2 && st.p.taps() == 1 && st.p.pad == 0 && use_mfma(st.p, b.dtype) && use_mfma(b.st[0].p, b.dtype) &&
            conv_mfma_dgrad_compact_addend_ok(b.st[0].p) && (dx || dry)) {
            ConvP pc = st.p;
            pc.H = st.p.Ho; pc.W = st.p.Wo; pc.stride = 1;
            TSM_TRY(run_conv_dgrad(pc, b.dtype, dyd, st.w, st.wd, dsc, nullptr, nullptr, ws, dry, sd));
            addend_stride = 2;
        } else {
            TSM_TRY(run_conv_dgrad(st.p, b.dtype, dyd, st.w, st.wd, dsc, nullptr, nullptr, ws, dry, sd));
        }
        if (ss) {
            if (hipEventRecord(ss->branch, ss->stream) != hipSuccess)
                return fail(TSM_ERR_LAUNCH, "block backward: cannot record the side stream's event");
            branch_open = true;
        }
        addend = dsc;
        return TSM_OK;
    };
    void* g = dyL;
    for (int i = L; i >= 1; --i) {
        StageDef& st = b.st[i];
        const ConvP& pp = b.st[i - 1].p;  // producer of this stage's input
        TSM_TRY(wgrad_beside(ss, &forked, st.p, b.dtype, b.z[i - 1], g, st.dw, st.dwp, acc_flag, ws, dry, s));
        if (i == L && b.proj) TSM_TRY(shortcut_dgrad());
        void* dzin = ws.take((size_t)pp.rows_out() * pp.Cout * es);
        // the ReLU mask and the BatchNorm reductions of the producing stage ride in the data gradient's
        // epilogue when its kernel can do that; otherwise they are a pass of their own
        const int nbf = conv_dgrad_fuse_blocks(st.p, b.dtype);
        const int nb = nbf ? nbf : red_blocks(pp.rows_out(), pp.Cout, b.dtype);
        float* part = ws.take_n<float>((size_t)nb * 2 * pp.Cout);
        float* coef = ws.take_n<float>(3 * (size_t)pp.Cout);
        if (nbf) {
            const DgradFuse fz = {(const bf16_t*)b.z[i - 1], (const bf16_t*)b.y[i - 1], b.bn[i - 1].mean, b.bn[i - 1].rstd, part};
            TSM_TRY(run_conv_dgrad(st.p, b.dtype, g, st.w, st.wd, dzin, nullptr, &fz, ws, dry, s));
        } else {
            TSM_TRY(run_conv_dgrad(st.p, b.dtype, g, st.w, st.wd, dzin, nullptr, nullptr, ws, dry, s));
            RUN(relu_bn_bwd_reduce(b.dtype, dzin, b.z[i - 1], b.y[i - 1], pp.rows_out(), pp.Cout, b.bn[i - 1].mean,
                                   b.bn[i - 1].rstd, dzin, part, nullptr, nullptr, nullptr, nullptr, s));
        }
        RUN(bn_bwd_coeffs(part, nb, pp.rows_out(), pp.Cout, b.bn[i - 1].mean, b.bn[i - 1].rstd, b.st[i - 1].g, coef,
                          b.st[i - 1].dg, b.st[i - 1].db, s));
        RUN(bn_bwd_apply(b.dtype, dzin, b.y[i - 1], pp.rows_out(), pp.Cout, coef, dzin, s));
        g = dzin;
    }
    TSM_TRY(wgrad_beside(ss, &forked, b.st[0].p, b.dtype, x, g, b.st[0].dw, b.st[0].dwp, acc_flag, ws, dry, s));
    if (b.proj) {
        StageDef& st = b.ds;
        TSM_TRY(wgrad_beside(ss, &forked, st.p, b.dtype, x, dyd, st.dw, st.dwp, acc_flag, ws, dry, s));
        if (branch_open && hipStreamWaitEvent(s, ss->branch, 0) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "block backward: cannot wait for the side stream");
    }
    if (dx || dry)
        TSM_TRY(run_conv_dgrad(b.st[0].p, b.dtype, g, b.st[0].w, b.st[0].wd, dx, addend, b.dx_fuse, ws, dry, s, addend_stride));
    return TSM_OK;
}

static void set_stage(StageDef& st, int F, int T, int H, int W, int Cin, int Cout, int KT, int k, int stride, int pad,
                      int fold) {
    st = StageDef{};
    ConvP& p = st.p;
    p.F = F; p.T = T; p.H = H; p.W = W; p.Cin = Cin; p.Cout = Cout; p.KT = KT; p.KH = k; p.KW = k;
    p.stride = stride; p.pad = pad; p.fold = fold;
    p.Ho = (H + 2 * pad - k) / stride + 1;
    p.Wo = (W + 2 * pad - k) / stride + 1;
}

int make_block_plan(const tsm_block_desc* d, BlockPlan* b, const char* who) {
    if (!d) return fail(TSM_ERR_NULLPTR, "%s: null descriptor", who);
    TSM_TRY(check_common(d->dtype, d->layout, who));
    if (d->N <= 0 || d->T <= 0 || d->Cin <= 0 || d->H <= 0 || d->W <= 0 || d->Cmid <= 0 || d->Cout <= 0 || d->stride <= 0)
        return fail(TSM_ERR_SHAPE, "%s: non-positive dimension", who);
    if (d->kind != TSM_BLOCK_BASIC && d->kind != TSM_BLOCK_BOTTLENECK && d->kind != TSM_BLOCK_BOTTLENECK_T3)
        return fail(TSM_ERR_UNSUPPORTED, "%s: unknown block kind %d", who, d->kind);
    if (!(d->bn_eps >= 0.f)) return fail(TSM_ERR_SHAPE, "%s: bn_eps must be >= 0", who);
    int fold = 0;
    const int fd = d->kind == TSM_BLOCK_BOTTLENECK_T3 ? 0 : d->fold_div;
    if (fold_of(d->Cin, fd, &fold) != TSM_OK) return fail(TSM_ERR_FOLD, "%s: invalid fold_div %d for Cin=%d", who, d->fold_div, d->Cin);
    *b = BlockPlan{};
    b->dtype = d->dtype;
    b->eps = d->bn_eps;
    b->bn_momentum = 0.f;
    const int F = d->N * d->T;
    if (d->kind == TSM_BLOCK_BASIC) {
        if (d->Cmid != d->Cin || d->Cout != d->Cin || d->stride != 1 || d->has_projection)
            return fail(TSM_ERR_SHAPE, "%s: the basic block needs Cmid == Cout == Cin, stride 1, no projection", who);
        b->nst = 2;
        set_stage(b->st[0], F, d->T, d->H, d->W, d->Cin, d->Cin, 1, 3, 1, 1, fold);
        set_stage(b->st[1], F, d->T, d->H, d->W, d->Cin, d->Cin, 1, 3, 1, 1, 0);
    } else {
        if (!d->has_projection && (d->Cout != d->Cin || d->stride != 1))
            return fail(TSM_ERR_SHAPE, "%s: an identity shortcut needs Cout == Cin and stride 1", who);
        if (d->H + 2 < 3 || d->W + 2 < 3) return fail(TSM_ERR_SHAPE, "%s: frame too small", who);
        b->nst = 3;
        const int KT = d->kind == TSM_BLOCK_BOTTLENECK_T3 ? 3 : 1;
        set_stage(b->st[0], F, d->T, d->H, d->W, d->Cin, d->Cmid, KT, 1, 1, 0, fold);
        set_stage(b->st[1], F, d->T, d->H, d->W, d->Cmid, d->Cmid, 1, 3, d->stride, 1, 0);
        set_stage(b->st[2], F, d->T, b->st[1].p.Ho, b->st[1].p.Wo, d->Cmid, d->Cout, 1, 1, 1, 0, 0);
        b->proj = d->has_projection != 0;
        if (b->proj) set_stage(b->ds, F, d->T, d->H, d->W, d->Cin, d->Cout, 1, 1, d->stride, 0, 0);
    }
    return TSM_OK;
}

static void bind_params(BlockPlan& b, const tsm_block_params* p, const tsm_block_grads* g) {
    const void* w[3] = {p->w1, p->w2, p->w3};
    const float* gm[3] = {p->g1, p->g2, p->g3};
    const float* bt[3] = {p->b1, p->b2, p->b3};
    for (int i = 0; i < b.nst; ++i) {
        b.st[i].w = w[i];
        b.st[i].g = gm[i];
        b.st[i].b = bt[i];
    }
    if (b.proj) {
        b.ds.w = p->wd;
        b.ds.g = p->gd;
        b.ds.b = p->bd;
    }
    if (g) {
        float* dw[3] = {g->dw1, g->dw2, g->dw3};
        float* dg[3] = {g->dg1, g->dg2, g->dg3};
        float* db[3] = {g->db1, g->db2, g->db3};
        for (int i = 0; i < b.nst; ++i) {
            b.st[i].dw = dw[i];
            b.st[i].dg = dg[i];
            b.st[i].db = db[i];
        }
        if (b.proj) {
            b.ds.dw = g->dwd;
            b.ds.dg = g->dgd;
            b.ds.db = g->dbd;
        }
    }
}

static int check_block_ptrs(const BlockPlan& b, bool bwd, const char* who) {
    for (int i = 0; i < b.nst; ++i) {
        if (!b.st[i].w || !b.st[i].g || !b.st[i].b) return fail(TSM_ERR_NULLPTR, "%s: null parameter pointer (stage %d)", who, i + 1);
        if (!aligned16(b.st[i].w)) return fail(TSM_ERR_ALIGN, "%s: weight pointers must be 16-byte aligned", who);
        if (bwd && (!b.st[i].dw || !b.st[i].dg || !b.st[i].db)) return fail(TSM_ERR_NULLPTR, "%s: null gradient pointer (stage %d)", who, i + 1);
    }
    if (b.proj) {
        if (!b.ds.w || !b.ds.g || !b.ds.b) return fail(TSM_ERR_NULLPTR, "%s: null projection parameter pointer", who);
        if (bwd && (!b.ds.dw || !b.ds.dg || !b.ds.db)) return fail(TSM_ERR_NULLPTR, "%s: null projection gradient pointer", who);
    }
    return TSM_OK;
}

static int block_entry(bool bwd, const tsm_block_desc* d, const void* x, const void* out_in, const void* dout,
                       const tsm_block_params* prm, void* out, void* saved, void* dx, const tsm_block_grads* grads,
                       void* wsp, size_t ws_bytes, bool dry, hipStream_t s, size_t* need_ws, size_t* need_saved) {
    const char* who = bwd ? "tsm_block_bwd" : "tsm_block_fwd";
    BlockPlan b;
    TSM_TRY(make_block_plan(d, &b, who));
    const bool tr = d->layout == TSM_NTCHW;
    if (!dry) {
        if (!prm) return fail(TSM_ERR_NULLPTR, "%s: null params", who);
        if (bwd && !grads) return fail(TSM_ERR_NULLPTR, "%s: null grads", who);
        bind_params(b, prm, grads);
        TSM_TRY(check_block_ptrs(b, bwd, who));
        if (!x || !saved || (!bwd && !out) || (bwd && (!out_in || !dout || !dx))) return fail(TSM_ERR_NULLPTR, "%s: null tensor pointer", who);
        if (!aligned16(x) || !aligned16(saved) || !aligned16(out) || !aligned16(out_in) || !aligned16(dout) || !aligned16(dx) || !aligned16(wsp))
            return fail(TSM_ERR_ALIGN, "%s: pointers must be 16-byte aligned", who);
        size_t req = 0;
        TSM_TRY(block_entry(bwd, d, x, out_in, dout, prm, out, saved, dx, grads, nullptr, 0, true, s, &req, nullptr));
        if (req > ws_bytes) return fail(TSM_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu", who, ws_bytes, req);
        if (req > 0 && !wsp) return fail(TSM_ERR_NULLPTR, "%s: null workspace", who);
    }
    Arena sv(dry ? nullptr : saved, (size_t)-1);
    block_saved_layout(b, sv, tr);
    if (need_saved) *need_saved = sv.used;
    Arena ws(dry ? nullptr : wsp, dry ? (size_t)-1 : ws_bytes);
    const int es = (int)dtype_size(d->dtype);
    const ConvP& p0 = b.st[0].p;
    const ConvP& pl = b.st[b.nst - 1].p;
    if (!bwd) {
        const void* xi = x;
        void* oi = out;
        if (tr) {
            RUN(transpose_frames(x, b.x_copy, p0.F, p0.Cin, p0.H * p0.W, es, s));
            xi = b.x_copy;
            oi = b.out_copy;
        }
        TSM_TRY(block_fwd_impl(b, xi, oi, ws, dry, s));
        if (tr) RUN(transpose_frames(oi, out, pl.F, pl.Ho * pl.Wo, pl.Cout, es, s));
    } else {
        const void *xi = x, *oi = out_in, *di = dout;
        void* dxi = dx;
        if (tr) {
            xi = b.x_copy;
            oi = b.out_copy;
            void* dt = ws.take((size_t)pl.rows_out() * pl.Cout * es);
            RUN(transpose_frames(dout, dt, pl.F, pl.Cout, pl.Ho * pl.Wo, es, s));
            di = dt;
            dxi = ws.take((size_t)p0.rows_in() * p0.Cin * es);
        }
        TSM_TRY(block_bwd_impl(b, xi, oi, di, dxi, ws, dry, s));
        if (tr) RUN(transpose_frames(dxi, dx, p0.F, p0.H * p0.W, p0.Cin, es, s));
    }
    if (need_ws) *need_ws = ws.used;
    return TSM_OK;
}

}  // namespace tsm

using namespace tsm;

extern "C" {

size_t tsm_conv_workspace_bytes(const tsm_conv_desc* d) {
    size_t best = 0;
    for (int which = 0; which < 3; ++which) {
        size_t need = 0;
        if (conv_entry(which, d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, 0, true, nullptr, &need) != TSM_OK) return 0;
        if (need > best) best = need;
    }
    return best;
}

int tsm_conv_fwd(const tsm_conv_desc* d, const void* x, const void* w, void* y, float* ch_sum, float* ch_sumsq,
                 void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(CONV_FWD, d, x, w, y, ch_sum, ch_sumsq, 0, ws, ws_bytes, false, (hipStream_t)stream, nullptr);
}

int tsm_conv_dgrad(const tsm_conv_desc* d, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes,
                   void* stream) {
    return conv_entry(CONV_DGRAD, d, dy, w, dx, nullptr, nullptr, 0, ws, ws_bytes, false, (hipStream_t)stream, nullptr);
}

int tsm_conv_wgrad(const tsm_conv_desc* d, const void* x, const void* dy, float* dw, int accumulate, void* ws,
                   size_t ws_bytes, void* stream) {
    return conv_entry(CONV_WGRAD, d, x, dy, dw, nullptr, nullptr, accumulate, ws, ws_bytes, false, (hipStream_t)stream, nullptr);
}

// ---- tsm_conv_fwd for callers that cannot allocate --------------------------------------------------------------
// The scratch of the forward convolution (the bf16 working copy of the weights, the per-block rows of the
// statistics epilogue, the transposed copies for the paper's memory order) lives in a device array that is part of
// the library's image: every GPU the library runs on holds its own copy, at its own address, until the process
// ends.  In host code the array's name only stands for the symbol; the device address comes from
// hipGetSymbolAddress, asked once per device with that device current, and only that address is handed to kernels.
static __device__ __align__(256) unsigned char g_noalloc_scratch[TSM_NOALLOC_SCRATCH_BYTES];

static int noalloc_scratch(void** out) {
    static void* ptr[16];               // per device; written once under the lock
    static std::mutex lock;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16)
        return fail(TSM_ERR_LAUNCH, "tsm_conv_fwd_noalloc: cannot tell the current device");
    std::lock_guard<std::mutex> hold(lock);
    if (!ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(TSM_ERR_LAUNCH, "tsm_conv_fwd_noalloc: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
        }
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return TSM_OK;
}

int tsm_conv_fwd_noalloc(const tsm_conv_desc* d, const void* x, const void* w, void* y, float* ch_sum, float* ch_sumsq,
                         void* stream) {
    size_t need = 0;
    TSM_TRY(conv_entry(CONV_FWD, d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, 0, true, nullptr, &need));
    if (need > (size_t)TSM_NOALLOC_SCRATCH_BYTES)
        return fail(TSM_ERR_WORKSPACE, "tsm_conv_fwd_noalloc: this convolution needs %zu bytes of scratch, the built-in buffer holds %zu",
                    need, (size_t)TSM_NOALLOC_SCRATCH_BYTES);
    // argument errors are reported before the device is touched
    if (!x || !w || !y) return fail(TSM_ERR_NULLPTR, "tsm_conv_fwd_noalloc: null tensor pointer");
    if ((ch_sum == nullptr) != (ch_sumsq == nullptr))
        return fail(TSM_ERR_NULLPTR, "tsm_conv_fwd_noalloc: ch_sum and ch_sumsq must both be set or both be NULL");
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return fail(TSM_ERR_ALIGN, "tsm_conv_fwd_noalloc: pointers must be 16-byte aligned");
    void* scratch = nullptr;
    TSM_TRY(noalloc_scratch(&scratch));
    // Nothing in the buffer has to start at zero: the packed weights and the transposed copies are written in full
    // before they are read, and every block of the convolution clears its own statistics row first.
    return conv_entry(CONV_FWD, d, x, w, y, ch_sum, ch_sumsq, 0, scratch, (size_t)TSM_NOALLOC_SCRATCH_BYTES, false,
                      (hipStream_t)stream, nullptr);
}

size_t tsm_block_infer_workspace_bytes(const tsm_block_desc* d) {
    size_t need = 0;
    if (block_infer_entry(d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, true, nullptr, &need) != TSM_OK) return 0;
    return need;
}

int tsm_block_infer(const tsm_block_desc* d, const void* x, const tsm_block_params* p, const tsm_block_stats* st, void* out,
                    void* ws, size_t ws_bytes, void* stream) {
    return block_infer_entry(d, x, p, st, out, ws, ws_bytes, false, (hipStream_t)stream, nullptr);
}

size_t tsm_block_saved_bytes(const tsm_block_desc* d) {
    size_t sv = 0;
    if (block_entry(false, d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, true,
                    nullptr, nullptr, &sv) != TSM_OK)
        return 0;
    return sv;
}

size_t tsm_block_workspace_bytes(const tsm_block_desc* d) {
    size_t a = 0, b = 0;
    if (block_entry(false, d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, true,
                    nullptr, &a, nullptr) != TSM_OK)
        return 0;
    if (block_entry(true, d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, true,
                    nullptr, &b, nullptr) != TSM_OK)
        return 0;
    return a > b ? a : b;
}

int tsm_block_fwd(const tsm_block_desc* d, const void* x, const tsm_block_params* p, void* out, void* saved, void* ws,
                  size_t ws_bytes, void* stream) {
    return block_entry(false, d, x, nullptr, nullptr, p, out, saved, nullptr, nullptr, ws, ws_bytes, false,
                       (hipStream_t)stream, nullptr, nullptr);
}

int tsm_block_bwd(const tsm_block_desc* d, const void* x, const void* out, const void* dout, const void* saved,
                  const tsm_block_params* p, void* dx, const tsm_block_grads* g, void* ws, size_t ws_bytes,
                  void* stream) {
    return block_entry(true, d, x, out, dout, p, nullptr, const_cast<void*>(saved), dx, g, ws, ws_bytes, false,
                       (hipStream_t)stream, nullptr, nullptr);
}

}  // extern "C"
