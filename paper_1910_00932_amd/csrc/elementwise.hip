// BatchNorm (training mode) / ReLU / residual-tail kernels and small utilities,
// channels-innermost frames [rows][C].  The paper names BatchNorm only in its
// training setting (section 4.1); the standard definition is used: batch mean
// and biased batch variance over all N*T frames, y_hat = (y-mean)*rstd,
// z = gamma*y_hat + beta.  All of these are HBM-bound: 16-byte vectors, one
// pass per tensor, per-channel reductions in registers -> LDS -> fp64 atomics.
#include "internal.h"

namespace tsm {

template <typename T, int V> struct alignas(sizeof(T) * V) Pack { T v[V]; };

// Stores of results that the caches cannot hold until their next use go past them (16-byte packs only).
template <typename T, int V>
__device__ __forceinline__ void store_pack(T* p, const Pack<T, V>& v, bool stream) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    if (sizeof(T) * V == 16 && stream)
        __builtin_nontemporal_store(*(const u32x4_t*)&v, (u32x4_t*)p);
    else
        *(Pack<T, V>*)p = v;
}
static inline bool stream_result(long rows, int C, int dtype) { return rows * C * (long)dtype_size(dtype) > (64L << 20); }

// ---------------------------------------------------------------------------------
// 16-byte stores over the aligned body, 4-byte stores over the (at most three) words in front of it and behind it.
__global__ void __launch_bounds__(256) fill_zero_kernel(uint32_t* p, int nhead, uint4* body, size_t n16, uint32_t* tail, int ntail) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) body[i] = make_uint4(0u, 0u, 0u, 0u);
    if (blockIdx.x == 0) {
        if ((int)threadIdx.x < nhead) p[threadIdx.x] = 0u;
        if ((int)threadIdx.x < ntail) tail[threadIdx.x] = 0u;
    }
}

// p: 4-byte aligned, bytes: a multiple of 4 (rounded up otherwise: every caller's buffer ends on a word)
int fill_zero(void* p, size_t bytes, hipStream_t s) {
    if (bytes == 0) return TSM_OK;
    size_t words = (bytes + 3) / 4;
    uint32_t* w = (uint32_t*)p;
    size_t nhead = ((16 - ((uintptr_t)p & 15)) & 15) / 4;
    if (nhead > words) nhead = words;
    words -= nhead;
    const size_t n16 = words / 4;
    const int ntail = (int)(words - n16 * 4);
    const size_t want = (n16 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 1 ? 1 : (want < 16384 ? want : 16384));
    fill_zero_kernel<<<dim3(blocks), dim3(256), 0, s>>>(w, (int)nhead, (uint4*)(w + nhead), n16, w + nhead + n16 * 4, ntail);
    return check_launch("fill_zero");
}

// ---- launch shape shared by every per-channel kernel ---------------------------------------
// Threads (tx, ty): tx walks channel vectors, ty walks rows; every thread keeps one
// channel vector for its whole life, so per-channel coefficients and partial sums
// stay in registers and consecutive lanes touch consecutive 16-byte pieces of a row.
struct RowShape {
    dim3 grid, block;
    int cv;
};

static RowShape row_shape(long rows, int C, int V, int rows_per_thread, int max_gx, int nt = 256) {
    RowShape r;
    r.cv = C / V;
    int bx = r.cv < nt ? r.cv : nt;
    int by = nt / bx;
    if (by < 1) by = 1;
    long gx = (rows + (long)by * rows_per_thread - 1) / ((long)by * rows_per_thread);
    if (gx < 1) gx = 1;
    if (gx > max_gx) gx = max_gx;
    r.block = dim3(bx, by);
    r.grid = dim3((unsigned)gx, (unsigned)((r.cv + bx - 1) / bx));
    return r;
}

static inline int vec_of(int dtype, int C) {
    const int v = dtype == TSM_F32 ? 4 : 8;
    return C % v == 0 ? v : 1;
}

static constexpr int RED_ROWS_PER_THREAD = 8, RED_MAX_GX = 512;
// Elementwise passes: one row per thread and 128-thread blocks (measured: a grid-stride loop over some twenty rows
// per thread costs 5 % on bn_bwd_apply and 10 % on the block tail, 256-thread blocks another 2 %).
static constexpr int EW_ROWS_PER_THREAD = 1, EW_MAX_GX = 1 << 22, EW_THREADS = 128;

// Number of per-block partial rows the reduction kernels write for this tensor.
int red_blocks(long rows, int C, int dtype) {
    return (int)row_shape(rows, C, vec_of(dtype, C), RED_ROWS_PER_THREAD, RED_MAX_GX).grid.x;
}

// Sums the per-thread partials a[V], b[V] over ty and stores them into this block's
// row of the partial buffer: prow[c] and prow[C + c].  No atomics: deterministic.
template <int V>
__device__ __forceinline__ void block_partial_2(const float* a, const float* b, int cvi, int cv, int C, float* prow) {
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
            prow[cvi * V + j] = sa;
            prow[C + cvi * V + j] = sb;
        }
    }
}

// ---- per-channel sum and sum of squares -------------------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) channel_stats_kernel(const T* __restrict__ y, long rows, int C, int cv,
                                                            float* __restrict__ partial) {
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
    block_partial_2<V>(s1, s2, cvi, cv, C, partial + (size_t)blockIdx.x * 2 * C);
}

template <typename T, int V>
static int channel_stats_tv(const T* y, long rows, int C, float* partial, hipStream_t s) {
    RowShape r = row_shape(rows, C, V, RED_ROWS_PER_THREAD, RED_MAX_GX);
    channel_stats_kernel<T, V><<<r.grid, r.block, 0, s>>>(y, rows, C, r.cv, partial);
    return check_launch("channel_stats");
}

// partial: fp32 [red_blocks(rows, C, dtype)][2*C]
int channel_stats(int dtype, const void* y, long rows, int C, float* partial, hipStream_t s) {
    const int v = vec_of(dtype, C);
    if (dtype == TSM_F32)
        return v == 4 ? channel_stats_tv<float, 4>((const float*)y, rows, C, partial, s)
                      : channel_stats_tv<float, 1>((const float*)y, rows, C, partial, s);
    return v == 8 ? channel_stats_tv<bf16_t, 8>((const bf16_t*)y, rows, C, partial, s)
                  : channel_stats_tv<bf16_t, 1>((const bf16_t*)y, rows, C, partial, s);
}

// Adds up the rows of a partial buffer for channel c = blockIdx.x*16 + threadIdx.x.  This kernel is pure latency (it
// sits between two dependent launches of every BatchNorm, forward and backward), so the rows are split over 64 ty
// lanes of a (16 x 64) block and a lane issues the loads of its first four rows together: up to 256 rows cost one
// memory round trip.  The lanes meet in a fixed order: the four ty lanes of a wavefront by two shuffles, the sixteen
// wavefronts through LDS.  The totals are valid on the threads with threadIdx.y == 0.
static constexpr int SP_C = 16, SP_R = 64;
__device__ __forceinline__ void sum_partials(const float* __restrict__ partial, int nblocks, int C, int c,
                                             double* out1, double* out2) {
    __shared__ double red[2][SP_R / 4][SP_C];
    double s1 = 0.0, s2 = 0.0;
    if (c < C) {
        float a[4] = {0.f, 0.f, 0.f, 0.f}, b[4] = {0.f, 0.f, 0.f, 0.f};
        for (int b0 = threadIdx.y; b0 < nblocks; b0 += 4 * SP_R) {
            float va[4], vb[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {   // rows beyond the end re-read the last row and count as zero: no branch around the loads
                const int r = b0 + k * SP_R;
                const size_t at = (size_t)(r < nblocks ? r : nblocks - 1) * 2 * C + c;
                va[k] = partial[at];
                vb[k] = partial[at + C];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool in = b0 + k * SP_R < nblocks;
                a[k] += in ? va[k] : 0.f;
                b[k] += in ? vb[k] : 0.f;
            }
        }
        s1 = ((double)a[0] + (double)a[1]) + ((double)a[2] + (double)a[3]);
        s2 = ((double)b[0] + (double)b[1]) + ((double)b[2] + (double)b[3]);
    }
    // thread (tx, ty) is lane (ty % 4) * 16 + tx of wavefront ty / 4
    s1 += __shfl_xor(s1, 16);
    s2 += __shfl_xor(s2, 16);
    s1 += __shfl_xor(s1, 32);
    s2 += __shfl_xor(s2, 32);
    if ((threadIdx.y & 3) == 0) {
        red[0][threadIdx.y >> 2][threadIdx.x] = s1;
        red[1][threadIdx.y >> 2][threadIdx.x] = s2;
    }
    __syncthreads();
    double t1 = 0.0, t2 = 0.0;
    if (threadIdx.y == 0) {
#pragma unroll
        for (int r = 0; r < SP_R / 4; ++r) {
            t1 += red[0][r][threadIdx.x];
            t2 += red[1][r][threadIdx.x];
        }
    }
    *out1 = t1;
    *out2 = t2;
}

// ---- partial statistics -> per-channel vectors ------------------------------------------------------
__global__ void __launch_bounds__(SP_C * SP_R) bn_finalize_kernel(const float* __restrict__ partial, int nblocks, double inv_m, double unbias, int C,
                                   const float* __restrict__ gamma, const float* __restrict__ beta, float eps,
                                   BnVec o, float* run_mean, float* run_var, float momentum) {
    const int c = blockIdx.x * SP_C + threadIdx.x;
    double s1, s2;
    sum_partials(partial, nblocks, C, c, &s1, &s2);
    if (c >= C || threadIdx.y != 0) return;
    const double mean = s1 * inv_m;
    double var = s2 * inv_m - mean * mean;
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

int bn_finalize(const float* partial, int nblocks, long rows, int C, const float* gamma, const float* beta, float eps,
                BnVec out, float* run_mean, float* run_var, float momentum, hipStream_t s) {
    const double inv_m = rows > 0 ? 1.0 / (double)rows : 0.0;
    const double unbias = rows > 1 ? (double)rows / (double)(rows - 1) : 1.0;
    bn_finalize_kernel<<<dim3(cdiv(C, SP_C)), dim3(SP_C, SP_R), 0, s>>>(partial, nblocks, inv_m, unbias, C, gamma, beta, eps,
                                                                out, run_mean, run_var, momentum);
    return check_launch("bn_finalize");
}

// Inference-mode BatchNorm as an affine map: scale = gamma / sqrt(var + eps), shift = beta - mean * scale.
__global__ void __launch_bounds__(256) bn_eval_vec_kernel(const float* __restrict__ gamma, const float* __restrict__ beta,
                                                          const float* __restrict__ mean, const float* __restrict__ var,
                                                          float eps, int C, float* __restrict__ scale,
                                                          float* __restrict__ shift) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    const float sc = gamma[c] / sqrtf(var[c] + eps);
    scale[c] = sc;
    shift[c] = fmaf(-mean[c], sc, beta[c]);
}

int bn_eval_vec(const float* gamma, const float* beta, const float* mean, const float* var, float eps, int C,
                float* scale, float* shift, hipStream_t s) {
    bn_eval_vec_kernel<<<dim3(cdiv(C, 256)), dim3(256), 0, s>>>(gamma, beta, mean, var, eps, C, scale, shift);
    return check_launch("bn_eval_vec");
}

__global__ void __launch_bounds__(SP_C * SP_R) stats_to_float_kernel(const float* __restrict__ partial, int nblocks, int C, float* sum, float* sumsq) {
    const int c = blockIdx.x * SP_C + threadIdx.x;
    double s1, s2;
    sum_partials(partial, nblocks, C, c, &s1, &s2);
    if (c >= C || threadIdx.y != 0) return;
    sum[c] = (float)s1;
    sumsq[c] = (float)s2;
}

int stats_to_float(const float* partial, int nblocks, int C, float* sum, float* sumsq, hipStream_t s) {
    stats_to_float_kernel<<<dim3(cdiv(C, SP_C)), dim3(SP_C, SP_R), 0, s>>>(partial, nblocks, C, sum, sumsq);
    return check_launch("stats_to_float");
}

// ---- z = relu(scale*y + shift) ------------------------------------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) bn_relu_kernel(const T* __restrict__ y, long rows, int C, int cv,
                                                      const float* __restrict__ scale,
                                                      const float* __restrict__ shift, T* __restrict__ z) {
    const int cvi = blockIdx.y * blockDim.x + threadIdx.x;
    if (cvi >= cv) return;
    float sc[V], sh[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        sc[j] = scale[cvi * V + j];
        sh[j] = shift[cvi * V + j];
    }
    for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < rows; r += (long)gridDim.x * blockDim.y) {
        const long off = r * C + (long)cvi * V;
        Pack<T, V> in = *(const Pack<T, V>*)(y + off), out;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float v = fmaf(Elem<T>::ld(in.v[j]), sc[j], sh[j]);
            out.v[j] = Elem<T>::st(v > 0.f ? v : 0.f);
        }
        *(Pack<T, V>*)(z + off) = out;
    }
}

template <typename T, int V>
static int bn_relu_tv(const T* y, long rows, int C, const float* scale, const float* shift, T* z, hipStream_t s) {
    RowShape r = row_shape(rows, C, V, EW_ROWS_PER_THREAD, EW_MAX_GX, EW_THREADS);
    bn_relu_kernel<T, V><<<r.grid, r.block, 0, s>>>(y, rows, C, r.cv, scale, shift, z);
    return check_launch("bn_relu_apply");
}

int bn_relu_apply(int dtype, const void* y, long rows, int C, const float* scale, const float* shift, void* z,
                  hipStream_t s) {
    if (rows == 0) return TSM_OK;
    const int v = vec_of(dtype, C);
    if (dtype == TSM_F32)
        return v == 4 ? bn_relu_tv<float, 4>((const float*)y, rows, C, scale, shift, (float*)z, s)
                      : bn_relu_tv<float, 1>((const float*)y, rows, C, scale, shift, (float*)z, s);
    return v == 8 ? bn_relu_tv<bf16_t, 8>((const bf16_t*)y, rows, C, scale, shift, (bf16_t*)z, s)
                  : bn_relu_tv<bf16_t, 1>((const bf16_t*)y, rows, C, scale, shift, (bf16_t*)z, s);
}

// ---- out = relu(scale*y + shift + shortcut') -------------------------------------------------------
template <typename T, int V, bool PROJ>
__global__ void __launch_bounds__(256) tail_kernel(const T* __restrict__ y, long rows, int C, int cv,
                                                   const float* __restrict__ scale, const float* __restrict__ shift,
                                                   const T* __restrict__ sc, const float* __restrict__ scale_d,
                                                   const float* __restrict__ shift_d, T* __restrict__ out, bool stream,
                                                   uint8_t* __restrict__ bits) {
    const int cvi = blockIdx.y * blockDim.x + threadIdx.x;
    if (cvi >= cv) return;
    float s0[V], h0[V], s1[V], h1[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        s0[j] = scale[cvi * V + j];
        h0[j] = shift[cvi * V + j];
        s1[j] = PROJ ? scale_d[cvi * V + j] : 1.f;
        h1[j] = PROJ ? shift_d[cvi * V + j] : 0.f;
    }
    for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < rows; r += (long)gridDim.x * blockDim.y) {
        const long off = r * C + (long)cvi * V;
        Pack<T, V> a = *(const Pack<T, V>*)(y + off), b = *(const Pack<T, V>*)(sc + off), o;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float rr = Elem<T>::ld(b.v[j]);
            if (PROJ) rr = fmaf(rr, s1[j], h1[j]);
            const float v = fmaf(Elem<T>::ld(a.v[j]), s0[j], h0[j]) + rr;
            o.v[j] = Elem<T>::st(v > 0.f ? v : 0.f);
        }
        store_pack<T, V>(out + off, o, stream);
        if (V == 8 && bits) {   // which of the eight stored values are positive: the ReLU decisions, one byte per vector
            unsigned m = 0;
#pragma unroll
            for (int j = 0; j < V; ++j) m |= (Elem<T>::ld(o.v[j]) > 0.f ? 1u : 0u) << j;
            bits[r * cv + cvi] = (uint8_t)m;
        }
    }
}

template <typename T, int V>
static int tail_tv(const T* y, long rows, int C, const float* scale, const float* shift, const T* sc,
                   const float* scale_d, const float* shift_d, T* out, uint8_t* bits, hipStream_t s) {
    RowShape r = row_shape(rows, C, V, EW_ROWS_PER_THREAD, EW_MAX_GX, EW_THREADS);
    const bool st = stream_result(rows, C, sizeof(T) == 2 ? TSM_BF16 : TSM_F32);
    if (scale_d)
        tail_kernel<T, V, true><<<r.grid, r.block, 0, s>>>(y, rows, C, r.cv, scale, shift, sc, scale_d, shift_d, out, st, bits);
    else
        tail_kernel<T, V, false><<<r.grid, r.block, 0, s>>>(y, rows, C, r.cv, scale, shift, sc, scale_d, shift_d, out, st, bits);
    return check_launch("block_tail_fwd");
}

bool block_tail_writes_bits(int dtype, int C) { return dtype == TSM_BF16 && C % 8 == 0; }

int block_tail_fwd(int dtype, const void* y, long rows, int C, const float* scale, const float* shift,
                   const void* shortcut, const float* scale_d, const float* shift_d, void* out, hipStream_t s,
                   uint8_t* out_bits) {
    if (rows == 0) return TSM_OK;
    const int v = vec_of(dtype, C);
    if (out_bits && !block_tail_writes_bits(dtype, C)) return fail(TSM_ERR_UNSUPPORTED, "block tail: decision bits need bf16 and channels % 8 == 0");
    if (dtype == TSM_F32)
        return v == 4 ? tail_tv<float, 4>((const float*)y, rows, C, scale, shift, (const float*)shortcut, scale_d, shift_d, (float*)out, nullptr, s)
                      : tail_tv<float, 1>((const float*)y, rows, C, scale, shift, (const float*)shortcut, scale_d, shift_d, (float*)out, nullptr, s);
    return v == 8 ? tail_tv<bf16_t, 8>((const bf16_t*)y, rows, C, scale, shift, (const bf16_t*)shortcut, scale_d, shift_d, (bf16_t*)out, out_bits, s)
                  : tail_tv<bf16_t, 1>((const bf16_t*)y, rows, C, scale, shift, (const bf16_t*)shortcut, scale_d, shift_d, (bf16_t*)out, nullptr, s);
}

// ---- backward, pass A: ReLU mask + the two BatchNorm reductions -------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) relu_bn_bwd_reduce_kernel(
    const T* __restrict__ dout, const T* __restrict__ act, const T* __restrict__ y, long rows, int C, int cv,
    const float* __restrict__ mean, const float* __restrict__ rstd, T* __restrict__ dz_out,
    float* __restrict__ partial, const T* __restrict__ y2, const float* __restrict__ mean2,
    const float* __restrict__ rstd2, float* __restrict__ partial2) {
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
            if (dz_out) *(Pack<T, V>*)(dz_out + off) = o;
        }
    }
    block_partial_2<V>(s1, s2, cvi, cv, C, partial + (size_t)blockIdx.x * 2 * C);
    if (y2) {
        __syncthreads();
        block_partial_2<V>(s1, s3, cvi, cv, C, partial2 + (size_t)blockIdx.x * 2 * C);
    }
}

template <typename T, int V>
static int relu_bn_bwd_reduce_tv(const T* dout, const T* act, const T* y, long rows, int C, const float* mean,
                                 const float* rstd, T* dz_out, float* partial, const T* y2, const float* mean2,
                                 const float* rstd2, float* partial2, hipStream_t s) {
    RowShape r = row_shape(rows, C, V, RED_ROWS_PER_THREAD, RED_MAX_GX);
    relu_bn_bwd_reduce_kernel<T, V><<<r.grid, r.block, 0, s>>>(dout, act, y, rows, C, r.cv, mean, rstd, dz_out, partial,
                                                                y2, mean2, rstd2, partial2);
    return check_launch("relu_bn_bwd_reduce");
}

// partial / partial2: fp32 [red_blocks(rows, C, dtype)][2*C]
int relu_bn_bwd_reduce(int dtype, const void* dout, const void* act, const void* y, long rows, int C,
                       const float* mean, const float* rstd, void* dz_out, float* partial, const void* y2,
                       const float* mean2, const float* rstd2, float* partial2, hipStream_t s) {
    if (rows == 0) return TSM_OK;
    const int v = vec_of(dtype, C);
#define TSM_RBR(T, V)                                                                                                \
    relu_bn_bwd_reduce_tv<T, V>((const T*)dout, (const T*)act, (const T*)y, rows, C, mean, rstd, (T*)dz_out, partial, \
                                (const T*)y2, mean2, rstd2, partial2, s)
    if (dtype == TSM_F32) return v == 4 ? TSM_RBR(float, 4) : TSM_RBR(float, 1);
    return v == 8 ? TSM_RBR(bf16_t, 8) : TSM_RBR(bf16_t, 1);
#undef TSM_RBR
}

// ---- backward, between the passes: sums -> per-channel coefficients ---------------------------------------
// dy = gamma*rstd*(dz - S1/m - yhat*S2/m), yhat = (y-mean)*rstd, rewritten as dy = a*dz + b*y + c with
//   a = gamma*rstd,  b = -gamma*rstd^2*S2/m,  c = gamma*rstd*(mean*rstd*S2/m - S1/m);
// dbeta = S1, dgamma = S2.
__global__ void __launch_bounds__(SP_C * SP_R) bn_bwd_coeffs_kernel(const float* __restrict__ partial, int nblocks, double inv_m, int C,
                                     const float* __restrict__ mean, const float* __restrict__ rstd,
                                     const float* __restrict__ gamma, float* __restrict__ coef,
                                     float* __restrict__ dgamma, float* __restrict__ dbeta) {
    const int c = blockIdx.x * SP_C + threadIdx.x;
    double s1, s2;
    sum_partials(partial, nblocks, C, c, &s1, &s2);
    if (c >= C || threadIdx.y != 0) return;
    const float g = gamma ? gamma[c] : 1.f;
    const float rs = rstd[c], mu = mean[c];
    const float m1 = (float)(s1 * inv_m), m2 = (float)(s2 * inv_m);
    coef[c] = g * rs;
    coef[C + c] = -g * rs * rs * m2;
    coef[2 * C + c] = g * rs * (mu * rs * m2 - m1);
    if (dbeta) dbeta[c] = (float)s1;
    if (dgamma) dgamma[c] = (float)s2;
}

int bn_bwd_coeffs(const float* partial, int nblocks, long rows, int C, const float* mean, const float* rstd,
                  const float* gamma, float* coef, float* dgamma, float* dbeta, hipStream_t s) {
    const double inv_m = rows > 0 ? 1.0 / (double)rows : 0.0;
    bn_bwd_coeffs_kernel<<<dim3(cdiv(C, SP_C)), dim3(SP_C, SP_R), 0, s>>>(partial, nblocks, inv_m, C, mean, rstd, gamma, coef,
                                                                  dgamma, dbeta);
    return check_launch("bn_bwd_coeffs");
}

// ---- backward, pass B: dy = a*dz + b*y + c ------------------------------------------------------------------
template <typename T, int V>
__global__ void __launch_bounds__(256) bn_bwd_apply_kernel(const T* __restrict__ dz, const T* __restrict__ y,
                                                           long rows, int C, int cv, const float* __restrict__ coef,
                                                           T* __restrict__ dy) {
    const int cvi = blockIdx.y * blockDim.x + threadIdx.x;
    if (cvi >= cv) return;
    float ka[V], kb[V], kc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        ka[j] = coef[cvi * V + j];
        kb[j] = coef[C + cvi * V + j];
        kc[j] = coef[2 * C + cvi * V + j];
    }
    for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < rows; r += (long)gridDim.x * blockDim.y) {
        const long off = r * C + (long)cvi * V;
        Pack<T, V> a = *(const Pack<T, V>*)(dz + off), b = *(const Pack<T, V>*)(y + off), o;
#pragma unroll
        for (int j = 0; j < V; ++j)
            o.v[j] = Elem<T>::st(fmaf(ka[j], Elem<T>::ld(a.v[j]), fmaf(kb[j], Elem<T>::ld(b.v[j]), kc[j])));
        *(Pack<T, V>*)(dy + off) = o;   // (read again right away by two kernels: a nontemporal store measured slower)
    }
}

template <typename T, int V>
static int bn_bwd_apply_tv(const T* dz, const T* y, long rows, int C, const float* coef, T* dy, hipStream_t s) {
    RowShape r = row_shape(rows, C, V, EW_ROWS_PER_THREAD, EW_MAX_GX, EW_THREADS);
    bn_bwd_apply_kernel<T, V><<<r.grid, r.block, 0, s>>>(dz, y, rows, C, r.cv, coef, dy);
    return check_launch("bn_bwd_apply");
}

// Two BatchNorms that share one upstream gradient (the last stage of a block and its projection shortcut):
// dy1 = a1*dz + b1*y1 + c1 and dy2 = a2*dz + b2*y2 + c2 from one read of dz.
template <typename T, int V>
__global__ void __launch_bounds__(256) bn_bwd_apply2_kernel(const T* __restrict__ dz, const T* __restrict__ y1,
                                                            const T* __restrict__ y2, long rows, int C, int cv,
                                                            const float* __restrict__ coef1, const float* __restrict__ coef2,
                                                            T* __restrict__ dy1, T* __restrict__ dy2) {
    const int cvi = blockIdx.y * blockDim.x + threadIdx.x;
    if (cvi >= cv) return;
    float ka[V], kb[V], kc[V], la[V], lb[V], lc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        ka[j] = coef1[cvi * V + j];
        kb[j] = coef1[C + cvi * V + j];
        kc[j] = coef1[2 * C + cvi * V + j];
        la[j] = coef2[cvi * V + j];
        lb[j] = coef2[C + cvi * V + j];
        lc[j] = coef2[2 * C + cvi * V + j];
    }
    for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < rows; r += (long)gridDim.x * blockDim.y) {
        const long off = r * C + (long)cvi * V;
        Pack<T, V> a = *(const Pack<T, V>*)(dz + off), b = *(const Pack<T, V>*)(y1 + off), c = *(const Pack<T, V>*)(y2 + off), o, p;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float g = Elem<T>::ld(a.v[j]);
            o.v[j] = Elem<T>::st(fmaf(ka[j], g, fmaf(kb[j], Elem<T>::ld(b.v[j]), kc[j])));
            p.v[j] = Elem<T>::st(fmaf(la[j], g, fmaf(lb[j], Elem<T>::ld(c.v[j]), lc[j])));
        }
        *(Pack<T, V>*)(dy1 + off) = o;
        *(Pack<T, V>*)(dy2 + off) = p;
    }
}

template <typename T, int V>
static int bn_bwd_apply2_tv(const T* dz, const T* y1, const T* y2, long rows, int C, const float* coef1, const float* coef2,
                            T* dy1, T* dy2, hipStream_t s) {
    RowShape r = row_shape(rows, C, V, EW_ROWS_PER_THREAD, EW_MAX_GX, EW_THREADS);
    bn_bwd_apply2_kernel<T, V><<<r.grid, r.block, 0, s>>>(dz, y1, y2, rows, C, r.cv, coef1, coef2, dy1, dy2);
    return check_launch("bn_bwd_apply");
}

int bn_bwd_apply2(int dtype, const void* dz, const void* y1, const float* coef1, void* dy1, const void* y2,
                  const float* coef2, void* dy2, long rows, int C, hipStream_t s) {
    if (rows == 0) return TSM_OK;
    const int v = vec_of(dtype, C);
    if (dtype == TSM_F32)
        return v == 4 ? bn_bwd_apply2_tv<float, 4>((const float*)dz, (const float*)y1, (const float*)y2, rows, C, coef1, coef2, (float*)dy1, (float*)dy2, s)
                      : bn_bwd_apply2_tv<float, 1>((const float*)dz, (const float*)y1, (const float*)y2, rows, C, coef1, coef2, (float*)dy1, (float*)dy2, s);
    return v == 8 ? bn_bwd_apply2_tv<bf16_t, 8>((const bf16_t*)dz, (const bf16_t*)y1, (const bf16_t*)y2, rows, C, coef1, coef2, (bf16_t*)dy1, (bf16_t*)dy2, s)
                  : bn_bwd_apply2_tv<bf16_t, 1>((const bf16_t*)dz, (const bf16_t*)y1, (const bf16_t*)y2, rows, C, coef1, coef2, (bf16_t*)dy1, (bf16_t*)dy2, s);
}

// coef: fp32 [3*C] from bn_bwd_coeffs
int bn_bwd_apply(int dtype, const void* dz, const void* y, long rows, int C, const float* coef, void* dy,
                 hipStream_t s) {
    if (rows == 0) return TSM_OK;
    const int v = vec_of(dtype, C);
    if (dtype == TSM_F32)
        return v == 4 ? bn_bwd_apply_tv<float, 4>((const float*)dz, (const float*)y, rows, C, coef, (float*)dy, s)
                      : bn_bwd_apply_tv<float, 1>((const float*)dz, (const float*)y, rows, C, coef, (float*)dy, s);
    return v == 8 ? bn_bwd_apply_tv<bf16_t, 8>((const bf16_t*)dz, (const bf16_t*)y, rows, C, coef, (bf16_t*)dy, s)
                  : bn_bwd_apply_tv<bf16_t, 1>((const bf16_t*)dz, (const bf16_t*)y, rows, C, coef, (bf16_t*)dy, s);
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
