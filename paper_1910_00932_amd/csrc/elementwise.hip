// BatchNorm (training mode) / ReLU / residual-tail kernels and small utilities,
// channels-innermost frames [rows][C].  The paper names BatchNorm only in its
// training setting (section 4.1); the standard definition is used: batch mean
// and biased batch variance over all N*T frames, y_hat = (y-mean)*rstd,
// z = gamma*y_hat + beta.  All of these are HBM-bound: 16-byte vectors, one
// pass per tensor, per-channel reductions in registers -> LDS -> fp64 atomics.
#include "internal.h"

namespace tsm {

template <typename T, int V> struct alignas(sizeof(T) * V) Pack { T v[V]; };

// ---------------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) p[i] = 0u;
}

int fill_zero(void* p, size_t bytes, hipStream_t s) {
    if (bytes == 0) return TSM_OK;
    size_t n = (bytes + 3) / 4;  // buffers come from 256-byte aligned arena slots
    unsigned blocks = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    fill_zero_kernel<<<dim3(blocks), dim3(256), 0, s>>>((uint32_t*)p, n);
    return check_launch("fill_zero");
}

// ---- row-reduction launch shape ------------------------------------------------------
// Threads (tx, ty): tx walks channel vectors, ty walks rows; every thread keeps
// one channel vector for its whole life, so partial sums stay in registers.
struct RedShape {
    dim3 grid, block;
    int cv;
};

static RedShape red_shape(long rows, int C, int V) {
    RedShape r;
    r.cv = C / V;
    int bx = r.cv < 256 ? r.cv : 256;
    int by = 256 / bx;
    if (by < 1) by = 1;
    long gx = (rows + (long)by * 8 - 1) / ((long)by * 8);  // >= 8 rows per thread
    if (gx < 1) gx = 1;
    if (gx > 2048) gx = 2048;
    r.block = dim3(bx, by);
    r.grid = dim3((unsigned)gx, (unsigned)((r.cv + bx - 1) / bx));
    return r;
}

// Sums the per-thread partials a[V], b[V] over ty and adds them into acc[c], acc[C+c].
template <int V>
__device__ __forceinline__ void block_reduce_2(float* a, float* b, int cvi, int cv, int C, double* acc) {
    __shared__ float red[2][256 * V];
    const int tx = threadIdx.x, ty = threadIdx.y, bx = blockDim.x, by = blockDim.y;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        red[0][(ty * bx + tx) * V + j] = a[j];
        red[1][(ty * bx + tx) * V + j] = b[j];
    }
    __syncthreads();
    if (ty == 0 && cvi < cv) {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float sa = 0.f, sb = 0.f;
            for (int r = 0; r < by; ++r) {
                sa += red[0][(r * bx + tx) * V + j];
                sb += red[1][(r * bx + tx) * V + j];
            }
            atomicAdd(acc + cvi * V + j, (double)sa);
            atomicAdd(acc + C + cvi * V + j, (double)sb);
        }
    }
}

// ---- per-channel sum and sum of squares -------------------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) channel_stats_kernel(const T* __restrict__ y, long rows, int C, int cv,
                                                            double* __restrict__ acc) {
    const int cvi = blockIdx.y * blockDim.x + threadIdx.x;
    float s1[V], s2[V];
#pragma unroll
    for (int j = 0; j < V; ++j) s1[j] = s2[j] = 0.f;
    if (cvi < cv) {
        for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < rows; r += (long)gridDim.x * blockDim.y) {
            Pack<T, V> pk = *(const Pack<T, V>*)(y + r * C + (long)cvi * V);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                float v = Elem<T>::ld(pk.v[j]);
                s1[j] += v;
                s2[j] = fmaf(v, v, s2[j]);
            }
        }
    }
    block_reduce_2<V>(s1, s2, cvi, cv, C, acc);
}

template <typename T>
static int channel_stats_t(const T* y, long rows, int C, double* acc, hipStream_t s) {
    constexpr int VEC = Elem<T>::VEC;
    if (C % VEC == 0) {
        RedShape r = red_shape(rows, C, VEC);
        channel_stats_kernel<T, VEC><<<r.grid, r.block, 0, s>>>(y, rows, C, r.cv, acc);
    } else {
        RedShape r = red_shape(rows, C, 1);
        channel_stats_kernel<T, 1><<<r.grid, r.block, 0, s>>>(y, rows, C, r.cv, acc);
    }
    return check_launch("channel_stats");
}

int channel_stats(int dtype, const void* y, long rows, int C, double* acc, hipStream_t s) {
    if (rows == 0) return TSM_OK;
    return dtype == TSM_F32 ? channel_stats_t<float>((const float*)y, rows, C, acc, s)
                            : channel_stats_t<bf16_t>((const bf16_t*)y, rows, C, acc, s);
}

// ---- statistics -> per-channel vectors ------------------------------------------------------
__global__ void bn_finalize_kernel(const double* __restrict__ acc, double inv_m, double unbias, int C,
                                   const float* __restrict__ gamma, const float* __restrict__ beta, float eps,
                                   BnVec o, float* run_mean, float* run_var, float momentum) {
    int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    const double mean = acc[c] * inv_m;
    double var = acc[C + c] * inv_m - mean * mean;
    if (var < 0) var = 0;
    const float rstd = (float)(1.0 / sqrt(var + (double)eps));
    const float g = gamma ? gamma[c] : 1.f;
    const float b = beta ? beta[c] : 0.f;
    o.mean[c] = (float)mean;
    o.rstd[c] = rstd;
    o.scale[c] = g * rstd;
    o.shift[c] = b - (float)mean * g * rstd;
    if (run_mean) {
        run_mean[c] = (1.f - momentum) * run_mean[c] + momentum * (float)mean;
        run_var[c] = (1.f - momentum) * run_var[c] + momentum * (float)(var * unbias);
    }
}

int bn_finalize(const double* acc, long rows, int C, const float* gamma, const float* beta, float eps, BnVec out,
                float* run_mean, float* run_var, float momentum, hipStream_t s) {
    const double inv_m = rows > 0 ? 1.0 / (double)rows : 0.0;
    const double unbias = rows > 1 ? (double)rows / (double)(rows - 1) : 1.0;
    bn_finalize_kernel<<<dim3(cdiv(C, 256)), dim3(256), 0, s>>>(acc, inv_m, unbias, C, gamma, beta, eps, out,
                                                               run_mean, run_var, momentum);
    return check_launch("bn_finalize");
}

__global__ void stats_to_float_kernel(const double* __restrict__ acc, int C, float* sum, float* sumsq) {
    int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    sum[c] = (float)acc[c];
    sumsq[c] = (float)acc[C + c];
}

int stats_to_float(const double* acc, int C, float* sum, float* sumsq, hipStream_t s) {
    stats_to_float_kernel<<<dim3(cdiv(C, 256)), dim3(256), 0, s>>>(acc, C, sum, sumsq);
    return check_launch("stats_to_float");
}

// ---- z = relu(scale*y + shift) ------------------------------------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) bn_relu_kernel(const T* __restrict__ y, size_t nvec, int cv,
                                                      const float* __restrict__ scale,
                                                      const float* __restrict__ shift, T* __restrict__ z) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= nvec) return;
    const int c0 = (int)(i % cv) * V;
    Pack<T, V> in = *(const Pack<T, V>*)(y + i * V), out;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        float v = fmaf(Elem<T>::ld(in.v[j]), scale[c0 + j], shift[c0 + j]);
        out.v[j] = Elem<T>::st(v > 0.f ? v : 0.f);
    }
    *(Pack<T, V>*)(z + i * V) = out;
}

template <typename T>
static int bn_relu_t(const T* y, long rows, int C, const float* scale, const float* shift, T* z, hipStream_t s) {
    constexpr int VEC = Elem<T>::VEC;
    if (C % VEC == 0) {
        size_t nvec = (size_t)rows * C / VEC;
        bn_relu_kernel<T, VEC><<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>(y, nvec, C / VEC, scale, shift, z);
    } else {
        size_t nvec = (size_t)rows * C;
        bn_relu_kernel<T, 1><<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>(y, nvec, C, scale, shift, z);
    }
    return check_launch("bn_relu_apply");
}

int bn_relu_apply(int dtype, const void* y, long rows, int C, const float* scale, const float* shift, void* z,
                  hipStream_t s) {
    if (rows == 0) return TSM_OK;
    return dtype == TSM_F32 ? bn_relu_t<float>((const float*)y, rows, C, scale, shift, (float*)z, s)
                            : bn_relu_t<bf16_t>((const bf16_t*)y, rows, C, scale, shift, (bf16_t*)z, s);
}

// ---- out = relu(scale*y + shift + shortcut') -------------------------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) tail_kernel(const T* __restrict__ y, size_t nvec, int cv,
                                                   const float* __restrict__ scale, const float* __restrict__ shift,
                                                   const T* __restrict__ sc, const float* __restrict__ scale_d,
                                                   const float* __restrict__ shift_d, T* __restrict__ out) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= nvec) return;
    const int c0 = (int)(i % cv) * V;
    Pack<T, V> a = *(const Pack<T, V>*)(y + i * V), b = *(const Pack<T, V>*)(sc + i * V), o;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        float r = Elem<T>::ld(b.v[j]);
        if (scale_d) r = fmaf(r, scale_d[c0 + j], shift_d[c0 + j]);
        float v = fmaf(Elem<T>::ld(a.v[j]), scale[c0 + j], shift[c0 + j]) + r;
        o.v[j] = Elem<T>::st(v > 0.f ? v : 0.f);
    }
    *(Pack<T, V>*)(out + i * V) = o;
}

template <typename T>
static int tail_t(const T* y, long rows, int C, const float* scale, const float* shift, const T* sc,
                  const float* scale_d, const float* shift_d, T* out, hipStream_t s) {
    constexpr int VEC = Elem<T>::VEC;
    if (C % VEC == 0) {
        size_t nvec = (size_t)rows * C / VEC;
        tail_kernel<T, VEC><<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>(y, nvec, C / VEC, scale, shift, sc, scale_d, shift_d, out);
    } else {
        size_t nvec = (size_t)rows * C;
        tail_kernel<T, 1><<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>(y, nvec, C, scale, shift, sc, scale_d, shift_d, out);
    }
    return check_launch("block_tail_fwd");
}

int block_tail_fwd(int dtype, const void* y, long rows, int C, const float* scale, const float* shift,
                   const void* shortcut, const float* scale_d, const float* shift_d, void* out, hipStream_t s) {
    if (rows == 0) return TSM_OK;
    return dtype == TSM_F32
               ? tail_t<float>((const float*)y, rows, C, scale, shift, (const float*)shortcut, scale_d, shift_d, (float*)out, s)
               : tail_t<bf16_t>((const bf16_t*)y, rows, C, scale, shift, (const bf16_t*)shortcut, scale_d, shift_d, (bf16_t*)out, s);
}

// ---- backward, pass A: ReLU mask + the two BatchNorm reductions -------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) relu_bn_bwd_reduce_kernel(
    const T* __restrict__ dout, const T* __restrict__ act, const T* __restrict__ y, long rows, int C, int cv,
    const float* __restrict__ mean, const float* __restrict__ rstd, T* __restrict__ dz_out, double* __restrict__ acc,
    const T* __restrict__ y2, const float* __restrict__ mean2, const float* __restrict__ rstd2,
    double* __restrict__ acc2) {
    const int cvi = blockIdx.y * blockDim.x + threadIdx.x;
    float s1[V], s2[V], s3[V], mu[V], rs[V], mu2[V], rs2[V];
#pragma unroll
    for (int j = 0; j < V; ++j) s1[j] = s2[j] = s3[j] = mu[j] = rs[j] = mu2[j] = rs2[j] = 0.f;
    if (cvi < cv) {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            mu[j] = mean[cvi * V + j];
            rs[j] = rstd[cvi * V + j];
            if (y2) {
                mu2[j] = mean2[cvi * V + j];
                rs2[j] = rstd2[cvi * V + j];
            }
        }
        for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < rows; r += (long)gridDim.x * blockDim.y) {
            const long off = r * C + (long)cvi * V;
            Pack<T, V> d = *(const Pack<T, V>*)(dout + off), a, yy = *(const Pack<T, V>*)(y + off), o, yy2;
            if (act) a = *(const Pack<T, V>*)(act + off);
            if (y2) yy2 = *(const Pack<T, V>*)(y2 + off);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float dz = (!act || Elem<T>::ld(a.v[j]) > 0.f) ? Elem<T>::ld(d.v[j]) : 0.f;
                o.v[j] = Elem<T>::st(dz);
                s1[j] += dz;
                s2[j] = fmaf(dz, (Elem<T>::ld(yy.v[j]) - mu[j]) * rs[j], s2[j]);
                if (y2) s3[j] = fmaf(dz, (Elem<T>::ld(yy2.v[j]) - mu2[j]) * rs2[j], s3[j]);
            }
            *(Pack<T, V>*)(dz_out + off) = o;
        }
    }
    block_reduce_2<V>(s1, s2, cvi, cv, C, acc);
    if (y2) {
        __syncthreads();
        block_reduce_2<V>(s1, s3, cvi, cv, C, acc2);
    }
}

template <typename T>
static int relu_bn_bwd_reduce_t(const T* dout, const T* act, const T* y, long rows, int C, const float* mean,
                                const float* rstd, T* dz_out, double* acc, const T* y2, const float* mean2,
                                const float* rstd2, double* acc2, hipStream_t s) {
    constexpr int VEC = Elem<T>::VEC;
    if (C % VEC == 0) {
        RedShape r = red_shape(rows, C, VEC);
        relu_bn_bwd_reduce_kernel<T, VEC><<<r.grid, r.block, 0, s>>>(dout, act, y, rows, C, r.cv, mean, rstd, dz_out, acc, y2, mean2, rstd2, acc2);
    } else {
        RedShape r = red_shape(rows, C, 1);
        relu_bn_bwd_reduce_kernel<T, 1><<<r.grid, r.block, 0, s>>>(dout, act, y, rows, C, r.cv, mean, rstd, dz_out, acc, y2, mean2, rstd2, acc2);
    }
    return check_launch("relu_bn_bwd_reduce");
}

int relu_bn_bwd_reduce(int dtype, const void* dout, const void* act, const void* y, long rows, int C,
                       const float* mean, const float* rstd, void* dz_out, double* acc, const void* y2,
                       const float* mean2, const float* rstd2, double* acc2, hipStream_t s) {
    if (rows == 0) return TSM_OK;
    return dtype == TSM_F32
               ? relu_bn_bwd_reduce_t<float>((const float*)dout, (const float*)act, (const float*)y, rows, C, mean, rstd,
                                             (float*)dz_out, acc, (const float*)y2, mean2, rstd2, acc2, s)
               : relu_bn_bwd_reduce_t<bf16_t>((const bf16_t*)dout, (const bf16_t*)act, (const bf16_t*)y, rows, C, mean,
                                              rstd, (bf16_t*)dz_out, acc, (const bf16_t*)y2, mean2, rstd2, acc2, s);
}

// ---- backward, pass B: dy = gamma*rstd*(dz - sum_dz/m - yhat*sum_dzyhat/m) -------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) bn_bwd_apply_kernel(const T* __restrict__ dz, const T* __restrict__ y,
                                                           size_t nvec, int cv, int C, float inv_m,
                                                           const float* __restrict__ mean,
                                                           const float* __restrict__ rstd,
                                                           const float* __restrict__ gamma,
                                                           const double* __restrict__ acc, T* __restrict__ dy,
                                                           float* __restrict__ dgamma, float* __restrict__ dbeta) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < (size_t)cv) {  // the first row's threads also publish dgamma / dbeta
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const int c = (int)i * V + j;
            if (dbeta) dbeta[c] = (float)acc[c];
            if (dgamma) dgamma[c] = (float)acc[C + c];
        }
    }
    if (i >= nvec) return;
    const int c0 = (int)(i % cv) * V;
    Pack<T, V> a = *(const Pack<T, V>*)(dz + i * V), b = *(const Pack<T, V>*)(y + i * V), o;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int c = c0 + j;
        const float rs = rstd[c];
        const float yhat = (Elem<T>::ld(b.v[j]) - mean[c]) * rs;
        const float sdz = (float)acc[c] * inv_m, sdzy = (float)acc[C + c] * inv_m;
        const float g = gamma ? gamma[c] : 1.f;
        o.v[j] = Elem<T>::st(g * rs * (Elem<T>::ld(a.v[j]) - sdz - yhat * sdzy));
    }
    *(Pack<T, V>*)(dy + i * V) = o;
}

template <typename T>
static int bn_bwd_apply_t(const T* dz, const T* y, long rows, int C, const float* mean, const float* rstd,
                          const float* gamma, const double* acc, T* dy, float* dgamma, float* dbeta, hipStream_t s) {
    constexpr int VEC = Elem<T>::VEC;
    const float inv_m = 1.f / (float)rows;
    if (C % VEC == 0) {
        size_t nvec = (size_t)rows * C / VEC;
        bn_bwd_apply_kernel<T, VEC><<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>(dz, y, nvec, C / VEC, C, inv_m, mean, rstd, gamma, acc, dy, dgamma, dbeta);
    } else {
        size_t nvec = (size_t)rows * C;
        bn_bwd_apply_kernel<T, 1><<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>(dz, y, nvec, C, C, inv_m, mean, rstd, gamma, acc, dy, dgamma, dbeta);
    }
    return check_launch("bn_bwd_apply");
}

int bn_bwd_apply(int dtype, const void* dz, const void* y, long rows, int C, const float* mean, const float* rstd,
                 const float* gamma, const double* acc, void* dy, float* dgamma, float* dbeta, hipStream_t s) {
    if (rows == 0) return TSM_OK;
    return dtype == TSM_F32 ? bn_bwd_apply_t<float>((const float*)dz, (const float*)y, rows, C, mean, rstd, gamma, acc,
                                                    (float*)dy, dgamma, dbeta, s)
                            : bn_bwd_apply_t<bf16_t>((const bf16_t*)dz, (const bf16_t*)y, rows, C, mean, rstd, gamma,
                                                     acc, (bf16_t*)dy, dgamma, dbeta, s);
}

// ---- out = a + b ------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) add_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ o,
                                                  size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) o[i] = Elem<T>::st(Elem<T>::ld(a[i]) + Elem<T>::ld(b[i]));
}

int add_tensors(int dtype, const void* a, const void* b, void* out, size_t n, hipStream_t s) {
    if (n == 0) return TSM_OK;
    unsigned blocks = (unsigned)((n + 255) / 256);
    if (dtype == TSM_F32)
        add_kernel<float><<<dim3(blocks), dim3(256), 0, s>>>((const float*)a, (const float*)b, (float*)out, n);
    else
        add_kernel<bf16_t><<<dim3(blocks), dim3(256), 0, s>>>((const bf16_t*)a, (const bf16_t*)b, (bf16_t*)out, n);
    return check_launch("add_tensors");
}

// ---- weight repacking ----------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) pack_fwd_kernel(const T* __restrict__ w, bf16_t* __restrict__ out, int Cout,
                                                       int Cin, int taps, int CinP) {
    long i = (long)blockIdx.x * 256 + threadIdx.x;  // out index: [co][tap][ci padded to CinP]
    if (i >= (long)Cout * CinP * taps) return;
    const int ci = (int)(i % CinP);
    const int tap = (int)((i / CinP) % taps);
    const int co = (int)(i / ((long)CinP * taps));
    out[i] = ci < Cin ? f32_to_bf16(Elem<T>::ld(w[((long)co * Cin + ci) * taps + tap])) : (bf16_t)0;
}

int pack_weights_fwd(int dtype, const void* w, bf16_t* out, int Cout, int Cin, int taps, int CinP, hipStream_t s) {
    long n = (long)Cout * CinP * taps;
    if (dtype == TSM_F32)
        pack_fwd_kernel<float><<<dim3(cdiv(n, 256)), dim3(256), 0, s>>>((const float*)w, out, Cout, Cin, taps, CinP);
    else
        pack_fwd_kernel<bf16_t><<<dim3(cdiv(n, 256)), dim3(256), 0, s>>>((const bf16_t*)w, out, Cout, Cin, taps, CinP);
    return check_launch("pack_weights_fwd");
}

template <typename T>
__global__ void __launch_bounds__(256) pack_dgrad_kernel(const T* __restrict__ w, bf16_t* __restrict__ out, int Cout,
                                                         int Cin, int KT, int KH, int KW) {
    const int taps = KT * KH * KW;
    long i = (long)blockIdx.x * 256 + threadIdx.x;  // out index: [ci][flipped tap][co]
    if (i >= (long)Cout * Cin * taps) return;
    const int co = (int)(i % Cout);
    const int ftap = (int)((i / Cout) % taps);
    const int ci = (int)(i / ((long)Cout * taps));
    const int kw = KW - 1 - ftap % KW, kh = KH - 1 - (ftap / KW) % KH, kt = KT - 1 - ftap / (KW * KH);
    const int tap = (kt * KH + kh) * KW + kw;
    out[i] = f32_to_bf16(Elem<T>::ld(w[((long)co * Cin + ci) * taps + tap]));
}

int pack_weights_dgrad(int dtype, const void* w, bf16_t* out, int Cout, int Cin, int KT, int KH, int KW,
                       hipStream_t s) {
    long n = (long)Cout * Cin * KT * KH * KW;
    if (dtype == TSM_F32)
        pack_dgrad_kernel<float><<<dim3(cdiv(n, 256)), dim3(256), 0, s>>>((const float*)w, out, Cout, Cin, KT, KH, KW);
    else
        pack_dgrad_kernel<bf16_t><<<dim3(cdiv(n, 256)), dim3(256), 0, s>>>((const bf16_t*)w, out, Cout, Cin, KT, KH, KW);
    return check_launch("pack_weights_dgrad");
}

__global__ void __launch_bounds__(256) unpack_wgrad_kernel(const float* __restrict__ packed, float* __restrict__ dw,
                                                           int Cout, int Cin, int taps, int CinP, int accumulate) {
    long i = (long)blockIdx.x * 256 + threadIdx.x;  // dw index: [co][ci][tap]
    if (i >= (long)Cout * Cin * taps) return;
    const int tap = (int)(i % taps);
    const int ci = (int)((i / taps) % Cin);
    const int co = (int)(i / ((long)Cin * taps));
    const float v = packed[((long)co * taps + tap) * CinP + ci];
    dw[i] = accumulate ? dw[i] + v : v;
}

int unpack_wgrad(const float* packed, float* dw, int Cout, int Cin, int taps, int CinP, int accumulate,
                 hipStream_t s) {
    long n = (long)Cout * Cin * taps;
    unpack_wgrad_kernel<<<dim3(cdiv(n, 256)), dim3(256), 0, s>>>(packed, dw, Cout, Cin, taps, CinP, accumulate);
    return check_launch("unpack_wgrad");
}

}  // namespace tsm
