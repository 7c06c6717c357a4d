// Plain one-thread-per-output convolution kernels, channels-innermost frames.
// They accept any shape and either storage type (fp32 accumulation) and serve
// the fp32 configurations and every shape the MFMA kernels do not take.
// Same definitions as the fast path: y = conv(S(x)), dx = S^T(conv^T(dy)),
// dw = sum dy (x) S(x) (paper section 2: shift + per-frame 2-D convolution).
#include "internal.h"

namespace tsm {

__device__ __forceinline__ int shift_dt(int c, int fold) { return c < fold ? 1 : (c < 2 * fold ? -1 : 0); }

template <typename T>
__global__ void __launch_bounds__(256) direct_fwd_kernel(ConvP p, const T* __restrict__ x, const T* __restrict__ w,
                                                         T* __restrict__ y, long total) {
    long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int co = (int)(idx % p.Cout);
    long m = idx / p.Cout;
    const int ow = (int)(m % p.Wo);
    m /= p.Wo;
    const int oh = (int)(m % p.Ho);
    const int f = (int)(m / p.Ho);
    const int t = f % p.T;
    const int taps = p.KT * p.KH * p.KW;
    float acc = 0.f;
    for (int kt = 0; kt < p.KT; ++kt) {
        const int df = kt - p.KT / 2;
        for (int kh = 0; kh < p.KH; ++kh) {
            const int ih = oh * p.stride + kh - p.pad;
            if (ih < 0 || ih >= p.H) continue;
            for (int kw = 0; kw < p.KW; ++kw) {
                const int iw = ow * p.stride + kw - p.pad;
                if (iw < 0 || iw >= p.W) continue;
                const int tap = (kt * p.KH + kh) * p.KW + kw;
                for (int ci = 0; ci < p.Cin; ++ci) {
                    const int d = df + shift_dt(ci, p.fold);
                    const int ts = t + d;
                    if (ts < 0 || ts >= p.T) continue;
                    const float xv = Elem<T>::ld(x[(((long)(f + d) * p.H + ih) * p.W + iw) * p.Cin + ci]);
                    const float wv = Elem<T>::ld(w[((long)co * p.Cin + ci) * taps + tap]);
                    acc = fmaf(xv, wv, acc);
                }
            }
        }
    }
    y[idx] = Elem<T>::st(acc);
}

template <typename T>
__global__ void __launch_bounds__(256) direct_dgrad_kernel(ConvP p, const T* __restrict__ dy,
                                                           const T* __restrict__ w, T* __restrict__ dx,
                                                           const T* __restrict__ addend, long total) {
    long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int ci = (int)(idx % p.Cin);
    long m = idx / p.Cin;
    const int iw = (int)(m % p.W);
    m /= p.W;
    const int ih = (int)(m % p.H);
    const int f = (int)(m / p.H);
    const int t = f % p.T;
    const int taps = p.KT * p.KH * p.KW;
    // S^T reads the un-shifted gradient of frame t - dt(ci)
    const int dsh = -shift_dt(ci, p.fold);
    float acc = 0.f;
    const int tsrc = t + dsh;
    if (tsrc >= 0 && tsrc < p.T) {
        for (int kt = 0; kt < p.KT; ++kt) {
            const int d = dsh - (kt - p.KT / 2);
            const int ty = t + d;
            if (ty < 0 || ty >= p.T) continue;
            for (int kh = 0; kh < p.KH; ++kh) {
                const int nh = ih + p.pad - kh;
                if (nh < 0 || nh % p.stride) continue;
                const int oh = nh / p.stride;
                if (oh >= p.Ho) continue;
                for (int kw = 0; kw < p.KW; ++kw) {
                    const int nw = iw + p.pad - kw;
                    if (nw < 0 || nw % p.stride) continue;
                    const int ow = nw / p.stride;
                    if (ow >= p.Wo) continue;
                    const int tap = (kt * p.KH + kh) * p.KW + kw;
                    const T* dyp = dy + (((long)(f + d) * p.Ho + oh) * p.Wo + ow) * p.Cout;
                    for (int co = 0; co < p.Cout; ++co)
                        acc = fmaf(Elem<T>::ld(dyp[co]), Elem<T>::ld(w[((long)co * p.Cin + ci) * taps + tap]), acc);
                }
            }
        }
    }
    if (addend) acc += Elem<T>::ld(addend[idx]);
    dx[idx] = Elem<T>::st(acc);
}

// One thread per weight element, one frame per blockIdx.y, fp32 atomics across frames.
template <typename T>
__global__ void __launch_bounds__(256) direct_wgrad_kernel(ConvP p, const T* __restrict__ x,
                                                           const T* __restrict__ dy, float* __restrict__ dw,
                                                           long total) {
    long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int taps = p.KT * p.KH * p.KW;
    const int tap = (int)(idx % taps);
    const int ci = (int)((idx / taps) % p.Cin);
    const int co = (int)(idx / ((long)taps * p.Cin));
    const int kw = tap % p.KW, kh = (tap / p.KW) % p.KH, kt = tap / (p.KW * p.KH);
    const int d = kt - p.KT / 2 + shift_dt(ci, p.fold);
    float total_acc = 0.f;
    for (int f = blockIdx.y; f < p.F; f += gridDim.y) {
        const int ts = f % p.T + d;
        if (ts < 0 || ts >= p.T) continue;
        float acc = 0.f;
        for (int oh = 0; oh < p.Ho; ++oh) {
            const int ih = oh * p.stride + kh - p.pad;
            if (ih < 0 || ih >= p.H) continue;
            for (int ow = 0; ow < p.Wo; ++ow) {
                const int iw = ow * p.stride + kw - p.pad;
                if (iw < 0 || iw >= p.W) continue;
                acc = fmaf(Elem<T>::ld(dy[(((long)f * p.Ho + oh) * p.Wo + ow) * p.Cout + co]),
                           Elem<T>::ld(x[(((long)(f + d) * p.H + ih) * p.W + iw) * p.Cin + ci]), acc);
            }
        }
        total_acc += acc;
    }
    atomicAdd(dw + idx, total_acc);
}

static int grid_for(long total, unsigned* blocks) {
    long b = (total + 255) / 256;
    if (b > 0x7fffffffL) return fail(TSM_ERR_SHAPE, "direct conv: problem too large");
    *blocks = (unsigned)b;
    return TSM_OK;
}

int conv_direct_fwd(const ConvP& p, int dtype, const void* x, const void* w, void* y, hipStream_t s) {
    const long total = p.rows_out() * p.Cout;
    if (total == 0) return TSM_OK;
    unsigned blocks;
    TSM_TRY(grid_for(total, &blocks));
    if (dtype == TSM_F32)
        direct_fwd_kernel<float><<<dim3(blocks), dim3(256), 0, s>>>(p, (const float*)x, (const float*)w, (float*)y, total);
    else
        direct_fwd_kernel<bf16_t><<<dim3(blocks), dim3(256), 0, s>>>(p, (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, total);
    return check_launch("conv_direct_fwd");
}

int conv_direct_dgrad(const ConvP& p, int dtype, const void* dy, const void* w, void* dx, const void* addend,
                      hipStream_t s) {
    const long total = p.rows_in() * p.Cin;
    if (total == 0) return TSM_OK;
    unsigned blocks;
    TSM_TRY(grid_for(total, &blocks));
    if (dtype == TSM_F32)
        direct_dgrad_kernel<float><<<dim3(blocks), dim3(256), 0, s>>>(p, (const float*)dy, (const float*)w, (float*)dx,
                                                                      (const float*)addend, total);
    else
        direct_dgrad_kernel<bf16_t><<<dim3(blocks), dim3(256), 0, s>>>(p, (const bf16_t*)dy, (const bf16_t*)w,
                                                                       (bf16_t*)dx, (const bf16_t*)addend, total);
    return check_launch("conv_direct_dgrad");
}

int conv_direct_wgrad(const ConvP& p, int dtype, const void* x, const void* dy, float* dw, hipStream_t s) {
    const long total = (long)p.Cout * p.Cin * p.taps();
    if (total == 0 || p.F == 0) return TSM_OK;
    unsigned blocks;
    TSM_TRY(grid_for(total, &blocks));
    const unsigned gy = (unsigned)(p.F < 64 ? p.F : 64);
    if (dtype == TSM_F32)
        direct_wgrad_kernel<float><<<dim3(blocks, gy), dim3(256), 0, s>>>(p, (const float*)x, (const float*)dy, dw, total);
    else
        direct_wgrad_kernel<bf16_t><<<dim3(blocks, gy), dim3(256), 0, s>>>(p, (const bf16_t*)x, (const bf16_t*)dy, dw, total);
    return check_launch("conv_direct_wgrad");
}

}  // namespace tsm
