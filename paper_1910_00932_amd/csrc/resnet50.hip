// One training iteration of TSM-ResNet-50 (paper section 3, model (3): ResNet-50
// backbone, the shift inserted into every residual block, 8 frames, no temporal
// pooling -- Table 2; Table 1: 24.3M parameters, 33G multiply-accumulates per
// clip, which fixes the stride on the 3x3 convolution; section 4.1: SGD with
// weight decay that skips BatchNorm and bias parameters).
//
// Everything between the clip tensor and the updated parameters runs here as a
// stream of kernel launches on the caller's stream, with no host synchronisation.
#include <string.h>
#include <algorithm>
#include <cmath>
#include <string>
#include <vector>
#include "block.h"
#include "internal.h"

namespace tsm {

// ---- parameter table -------------------------------------------------------------------
struct TensorInfo {
    std::string name;
    int64_t offset;
    int ndim;
    int shape[4];
    bool decays;
    int64_t count() const {
        int64_t n = 1;
        for (int i = 0; i < ndim; ++i) n *= shape[i];
        return n;
    }
};

struct StageSpec { const char* name; int blocks, mid, stride; };
static const StageSpec kStages[4] = {{"res2", 3, 64, 1}, {"res3", 4, 128, 2}, {"res4", 6, 256, 2}, {"res5", 3, 512, 2}};

static std::vector<TensorInfo> build_table(int num_classes) {
    std::vector<TensorInfo> t;
    int64_t off = 0;
    auto add = [&](const std::string& name, std::initializer_list<int> shp, bool decays) {
        TensorInfo ti;
        ti.name = name;
        ti.offset = off;
        ti.ndim = (int)shp.size();
        int i = 0;
        for (int v : shp) ti.shape[i++] = v;
        for (; i < 4; ++i) ti.shape[i] = 1;
        ti.decays = decays;
        off += ti.count();
        t.push_back(ti);
    };
    auto add_bn = [&](const std::string& pre, int c) {
        add(pre + ".g", {c}, false);
        add(pre + ".b", {c}, false);
    };
    add("conv1.w", {64, 3, 7, 7}, true);
    add_bn("bn1", 64);
    int cin = 64;
    for (const StageSpec& st : kStages) {
        for (int b = 0; b < st.blocks; ++b) {
            const std::string pre = std::string(st.name) + "." + std::to_string(b) + ".";
            add(pre + "c1.w", {st.mid, cin, 1, 1}, true);
            add_bn(pre + "bn1", st.mid);
            add(pre + "c2.w", {st.mid, st.mid, 3, 3}, true);
            add_bn(pre + "bn2", st.mid);
            add(pre + "c3.w", {4 * st.mid, st.mid, 1, 1}, true);
            add_bn(pre + "bn3", 4 * st.mid);
            if (b == 0) {
                add(pre + "ds.w", {4 * st.mid, cin, 1, 1}, true);
                add_bn(pre + "dsbn", 4 * st.mid);
            }
            cin = 4 * st.mid;
        }
    }
    add("fc.w", {num_classes, 2048}, true);
    add("fc.b", {num_classes}, false);
    return t;
}

static int find_tensor(const std::vector<TensorInfo>& t, const std::string& name) {
    for (size_t i = 0; i < t.size(); ++i)
        if (t[i].name == name) return (int)i;
    return -1;
}

// ---- stem in space-to-depth form ------------------------------------------------------------------
// The 7x7 stride-2 convolution over 3 channels equals a 4x4 stride-1 convolution over the 2x2
// space-to-depth image of the zero-padded input: with xs[h][w][(ph, pw, c)] = x[2h+ph-3][2w+pw-3][c],
//   y[oh][ow] = sum over th, tw < 4, ph, pw < 2, c of w[2th+ph][2tw+pw][c] * xs[oh+th][ow+tw][(ph, pw, c)]
// (taps with index 7 are zero).  xs keeps 16 values per pixel (channel (ph*2+pw)*4 + c, c = 3 is zero), so the
// four taps along W of one output pixel are 64 contiguous values: the MFMA kernels see a convolution with
// KH = 4, KW = 1, 64 channels and a pixel pitch of 16.  Every tap lies inside xs (S/2 + 3 pixels each way).
__global__ void __launch_bounds__(256) clips_to_s2d_kernel(const bf16_t* __restrict__ in, uint4* __restrict__ out,
                                                           int S, int Hs, long total) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;   // output pixel
    if (i >= total) return;
    const int w = (int)(i % Hs), h = (int)((i / Hs) % Hs);
    const long f = i / ((long)Hs * Hs);
    const bf16_t* base = in + f * 3 * (long)S * S;
    uint32_t v[8];
#pragma unroll
    for (int sp = 0; sp < 4; ++sp) {
        const int r = 2 * h + (sp >> 1) - 3, q = 2 * w + (sp & 1) - 3;
        uint32_t c0 = 0, c1 = 0, c2 = 0;
        if (r >= 0 && r < S && q >= 0 && q < S) {
            const bf16_t* px = base + (long)r * S + q;
            c0 = px[0]; c1 = px[(long)S * S]; c2 = px[2 * (long)S * S];
        }
        v[2 * sp] = c0 | (c1 << 16);
        v[2 * sp + 1] = c2;
    }
    out[2 * i] = make_uint4(v[0], v[1], v[2], v[3]);
    out[2 * i + 1] = make_uint4(v[4], v[5], v[6], v[7]);
}

// k index of the space-to-depth weights [64][4 th][4 tw][(ph, pw, c)] for (kh, kw, c)
__device__ __forceinline__ int s2d_index(int kh, int kw, int c) {
    return (kh >> 1) * 64 + (kw >> 1) * 16 + (((kh & 1) * 2 + (kw & 1)) * 4) + c;
}
__global__ void __launch_bounds__(256) stem_pack_kernel(const float* __restrict__ w, bf16_t* __restrict__ out) {
    const int co = blockIdx.x, k = threadIdx.x;   // one output channel per block, one packed element per thread
    const int th = k >> 6, tw = (k >> 4) & 3, sp = (k >> 2) & 3, c = k & 3;
    const int kh = 2 * th + (sp >> 1), kw = 2 * tw + (sp & 1);
    float v = 0.f;
    if (kh < 7 && kw < 7 && c < 3) v = w[((co * 3 + c) * 7 + kh) * 7 + kw];
    out[co * 256 + k] = f32_to_bf16(v);
}
// dw [64][3][7][7] += packed gradient [64][256]
__global__ void __launch_bounds__(256) stem_unpack_kernel(const float* __restrict__ packed, float* __restrict__ dw) {
    const int co = blockIdx.x, e = threadIdx.x;
    if (e >= 147) return;
    const int c = e / 49, kh = (e / 7) % 7, kw = e % 7;
    dw[co * 147 + e] += packed[co * 256 + s2d_index(kh, kw, c)];
}

// ---- BN + ReLU + 3x3/2 max-pool (padding 1; padding never wins) ---------------------------------
// Values are rounded to bf16 before they are compared, so the first-maximum rule is
// applied to the tensor a separate BN/ReLU pass would have stored.
template <typename T>
__global__ void __launch_bounds__(256) stem_pool_fwd_kernel(const T* __restrict__ y, const float* __restrict__ scale,
                                                            const float* __restrict__ shift, T* __restrict__ out,
                                                            uint8_t* __restrict__ arg, int H, int W, int Ho, int Wo,
                                                            int cv, long total) {
    constexpr int V = Elem<T>::VEC;
    long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int v = (int)(i % cv);
    long r = i / cv;
    const int ow = (int)(r % Wo);
    r /= Wo;
    const int oh = (int)(r % Ho);
    const long f = r / Ho;
    float best[V], sc[V], sh[V];
    int barg[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        best[j] = -1.f;   // post-ReLU values are >= 0, so any valid tap beats this
        barg[j] = 0;
        sc[j] = scale[v * V + j];
        sh[j] = shift[v * V + j];
    }
    for (int kh = 0; kh < 3; ++kh) {
        const int ih = 2 * oh + kh - 1;
        if (ih < 0 || ih >= H) continue;
        for (int kw = 0; kw < 3; ++kw) {
            const int iw = 2 * ow + kw - 1;
            if (iw < 0 || iw >= W) continue;
            const Vec16<T> pk = *(const Vec16<T>*)(y + ((f * H + ih) * W + iw) * (long)cv * V + v * V);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                float z = fmaf(Elem<T>::ld(pk.v[j]), sc[j], sh[j]);
                z = Elem<T>::ld(Elem<T>::st(z > 0.f ? z : 0.f));
                if (z > best[j]) {
                    best[j] = z;
                    barg[j] = kh * 3 + kw;
                }
            }
        }
    }
    Vec16<T> o;
    uint8_t ab[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        o.v[j] = Elem<T>::st(best[j]);
        ab[j] = (uint8_t)barg[j];
    }
    if (V == 8) *(uint2*)(arg + i * V) = *(const uint2*)ab;
    else *(uint32_t*)(arg + i * V) = *(const uint32_t*)ab;
    *(Vec16<T>*)(out + i * V) = o;
}

// Gradient of the pooled tensor routed back to the window position that won, times the ReLU mask of the
// (recomputed) stem activation: dz, stored to `da`.  Gather form: no atomics.  The same pass accumulates the
// two BatchNorm-backward sums of dz (as stored), one row of `partial` per block, in a fixed order.
// Block (C/V, 256/(C/V)): thread x = channel vector, thread y = row lane; rows are conv-output pixels.
template <typename T>
__global__ void __launch_bounds__(256) stem_pool_bwd_kernel(const T* __restrict__ dp, const uint8_t* __restrict__ arg,
                                                            const T* __restrict__ y, const float* __restrict__ scale,
                                                            const float* __restrict__ shift, const float* __restrict__ mean,
                                                            const float* __restrict__ rstd, T* __restrict__ da,
                                                            float* __restrict__ partial, int H, int W, int Ho, int Wo,
                                                            long rows) {
    constexpr int V = Elem<T>::VEC, C = 64, cv = C / V;
    const int v = threadIdx.x;
    float sc[V], sh[V], mu[V], rs[V], s1[V], s2[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        sc[j] = scale[v * V + j];
        sh[j] = shift[v * V + j];
        mu[j] = mean[v * V + j];
        rs[j] = rstd[v * V + j];
        s1[j] = s2[j] = 0.f;
    }
    for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < rows; r += (long)gridDim.x * blockDim.y) {
        const int iw = (int)(r % W), ih = (int)((r / W) % H);
        const long f = r / ((long)W * H);
        float g[V];
#pragma unroll
        for (int j = 0; j < V; ++j) g[j] = 0.f;
        // windows [2*oh-1, 2*oh+1] containing ih: one (even ih) or two (odd ih), likewise along w.  All four
        // candidates are loaded without branches (clamped to a valid window, duplicates and windows beyond the
        // border get a code that no winner has), so that their latencies overlap.
        const int oh0 = ih / 2, oh1 = (ih + 1) / 2, ow0 = iw / 2, ow1 = (iw + 1) / 2;
        const bool vh0 = oh0 < Ho, vh1 = oh1 != oh0 && oh1 < Ho, vw0 = ow0 < Wo, vw1 = ow1 != ow0 && ow1 < Wo;
        const int ch0 = oh0 < Ho ? oh0 : Ho - 1, ch1 = oh1 < Ho ? oh1 : Ho - 1;
        const int cw0 = ow0 < Wo ? ow0 : Wo - 1, cw1 = ow1 < Wo ? ow1 : Wo - 1;
        const int kh0 = ih - (2 * oh0 - 1), kh1 = ih - (2 * oh1 - 1), kw0 = iw - (2 * ow0 - 1), kw1 = iw - (2 * ow1 - 1);
        const long fo = f * Ho;
        const long o00 = ((fo + ch0) * Wo + cw0) * (long)cv + v, o01 = ((fo + ch0) * Wo + cw1) * (long)cv + v;
        const long o10 = ((fo + ch1) * Wo + cw0) * (long)cv + v, o11 = ((fo + ch1) * Wo + cw1) * (long)cv + v;
        const int code[4] = {vh0 && vw0 ? kh0 * 3 + kw0 : 255, vh0 && vw1 ? kh0 * 3 + kw1 : 255,
                             vh1 && vw0 ? kh1 * 3 + kw0 : 255, vh1 && vw1 ? kh1 * 3 + kw1 : 255};
        const long off[4] = {o00, o01, o10, o11};
        Vec16<T> dq[4];
        uint8_t aq[4][V];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            dq[q] = *(const Vec16<T>*)(dp + off[q] * V);
            if (V == 8) *(uint2*)aq[q] = *(const uint2*)(arg + off[q] * V);
            else *(uint32_t*)aq[q] = *(const uint32_t*)(arg + off[q] * V);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < V; ++j)
                if ((int)aq[q][j] == code[q]) g[j] += Elem<T>::ld(dq[q].v[j]);
        const long i = r * cv + v;
        const Vec16<T> pk = *(const Vec16<T>*)(y + i * V);
        Vec16<T> o;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float yv = Elem<T>::ld(pk.v[j]);
            const float z = fmaf(yv, sc[j], sh[j]);
            const bool live = Elem<T>::ld(Elem<T>::st(z > 0.f ? z : 0.f)) > 0.f;
            o.v[j] = Elem<T>::st(live ? g[j] : 0.f);
            const float dz = Elem<T>::ld(o.v[j]);
            s1[j] += dz;
            s2[j] = fmaf(dz, (yv - mu[j]) * rs[j], s2[j]);
        }
        *(Vec16<T>*)(da + i * V) = o;
    }
    __shared__ float red[2][256 * V];
    const int t = threadIdx.y * cv + v;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        red[0][t * V + j] = s1[j];
        red[1][t * V + j] = s2[j];
    }
    __syncthreads();
    if (threadIdx.y == 0) {
        float* prow = partial + (size_t)blockIdx.x * 2 * C;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float sa = 0.f, sb = 0.f;
            for (int q = 0; q < (int)blockDim.y; ++q) {
                sa += red[0][(q * cv + v) * V + j];
                sb += red[1][(q * cv + v) * V + j];
            }
            prow[v * V + j] = sa;
            prow[C + v * V + j] = sb;
        }
    }
}

// The same for even H and W, one 2 x 2 patch of conv-output pixels per thread and pass: the patch (2a.., 2b..) lies in
// the pooling windows (a, b), (a, b+1), (a+1, b), (a+1, b+1) only, so four window loads serve four pixels (the
// one-pixel form loads four windows per pixel).  Window (oh, ow) covers rows 2*oh-1 .. 2*oh+1: the code kh*3 + kw of
// a pixel inside a window follows from its position in the patch.
template <typename T>
__global__ void __launch_bounds__(256) stem_pool_bwd_patch_kernel(const T* __restrict__ dp, const uint8_t* __restrict__ arg,
                                                                  const T* __restrict__ y, const float* __restrict__ scale,
                                                                  const float* __restrict__ shift, const float* __restrict__ mean,
                                                                  const float* __restrict__ rstd, T* __restrict__ da,
                                                                  float* __restrict__ partial, int H, int W, int Ho, int Wo,
                                                                  long patches) {
    constexpr int V = Elem<T>::VEC, C = 64, cv = C / V;
    const int v = threadIdx.x;
    float sc[V], sh[V], mu[V], rs[V], s1[V], s2[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        sc[j] = scale[v * V + j];
        sh[j] = shift[v * V + j];
        mu[j] = mean[v * V + j];
        rs[j] = rstd[v * V + j];
        s1[j] = s2[j] = 0.f;
    }
    const int H2 = H / 2, W2 = W / 2;
    for (long r = (long)blockIdx.x * blockDim.y + threadIdx.y; r < patches; r += (long)gridDim.x * blockDim.y) {
        const int b = (int)(r % W2), a = (int)((r / W2) % H2);
        const long f = r / ((long)W2 * H2);
        // windows w = 2*dh + dw at (a + dh, b + dw); those beyond the border are clamped for the load and get a code
        // that no winner has
        const bool vh[2] = {a < Ho, a + 1 < Ho}, vw[2] = {b < Wo, b + 1 < Wo};
        Vec16<T> dq[4];
        uint8_t aq[4][V];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int oh = a + (w >> 1), ow = b + (w & 1);
            const long o = (((f * Ho) + (oh < Ho ? oh : Ho - 1)) * Wo + (ow < Wo ? ow : Wo - 1)) * (long)cv + v;
            dq[w] = *(const Vec16<T>*)(dp + o * V);
            if (V == 8) *(uint2*)aq[w] = *(const uint2*)(arg + o * V);
            else *(uint32_t*)aq[w] = *(const uint32_t*)(arg + o * V);
        }
        Vec16<T> pk[4];
#pragma unroll
        for (int p = 0; p < 4; ++p)
            pk[p] = *(const Vec16<T>*)(y + (((f * H + 2 * a + (p >> 1)) * W + 2 * b + (p & 1)) * (long)cv + v) * V);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int ph = p >> 1, pw = p & 1;      // pixel (2a + ph, 2b + pw)
            float g[V];
#pragma unroll
            for (int j = 0; j < V; ++j) g[j] = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const int dh = w >> 1, dw = w & 1;
                // rows of window a + dh: 2a + 2dh - 1 .. 2a + 2dh + 1; the pixel's row 2a + ph lies inside iff
                // kh = ph + 1 - 2dh is in 0..2 (ph = 0 is outside the lower window), likewise along w
                const int kh = ph + 1 - 2 * dh, kw = pw + 1 - 2 * dw;
                if (kh < 0 || kw < 0) continue;      // (compile-time: p, w are unrolled)
                const int code = vh[dh] && vw[dw] ? kh * 3 + kw : 255;
#pragma unroll
                for (int j = 0; j < V; ++j)
                    if ((int)aq[w][j] == code) g[j] += Elem<T>::ld(dq[w].v[j]);
            }
            Vec16<T> o;
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float yv = Elem<T>::ld(pk[p].v[j]);
                const float z = fmaf(yv, sc[j], sh[j]);
                const bool live = Elem<T>::ld(Elem<T>::st(z > 0.f ? z : 0.f)) > 0.f;
                o.v[j] = Elem<T>::st(live ? g[j] : 0.f);
                const float dz = Elem<T>::ld(o.v[j]);
                s1[j] += dz;
                s2[j] = fmaf(dz, (yv - mu[j]) * rs[j], s2[j]);
            }
            *(Vec16<T>*)(da + (((f * H + 2 * a + ph) * W + 2 * b + pw) * (long)cv + v) * V) = o;
        }
    }
    __shared__ float red[2][256 * V];
    const int t = threadIdx.y * cv + v;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        red[0][t * V + j] = s1[j];
        red[1][t * V + j] = s2[j];
    }
    __syncthreads();
    if (threadIdx.y == 0) {
        float* prow = partial + (size_t)blockIdx.x * 2 * C;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float sa = 0.f, sb = 0.f;
            for (int q = 0; q < (int)blockDim.y; ++q) {
                sa += red[0][(q * cv + v) * V + j];
                sb += red[1][(q * cv + v) * V + j];
            }
            prow[v * V + j] = sa;
            prow[C + v * V + j] = sb;
        }
    }
}

// ---- head: global average pool + temporal consensus + linear + softmax cross-entropy ---------
// The consensus (mean over T of the per-frame linear outputs) is an affine map, so the
// mean over frames and pixels is taken first: pm[n][c] = mean_{t,h,w} feat[n,t,h,w,c].
// Block = 32 channel vectors x 8 row lanes: 16-byte loads, the eight row lanes meet in LDS in a fixed order.
template <typename T>
__global__ void __launch_bounds__(256) pool_mean_kernel(const T* __restrict__ feat, float* __restrict__ pm,
                                                        int rows_per_clip, int C) {
    constexpr int V = Elem<T>::VEC;
    __shared__ float red[8][32 * V];
    const int n = blockIdx.y;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c0 = (blockIdx.x * 32 + tx) * V;
    float acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = 0.f;
    if (c0 < C) {
        const T* p = feat + (long)n * rows_per_clip * C + c0;
        for (int r = ty; r < rows_per_clip; r += 8) {
            const Vec16<T> v = *(const Vec16<T>*)(p + (long)r * C);
#pragma unroll
            for (int j = 0; j < V; ++j) acc[j] += Elem<T>::ld(v.v[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < V; ++j) red[ty][tx * V + j] = acc[j];
    __syncthreads();
    const int col = threadIdx.x;
    if (col < 32 * V && blockIdx.x * 32 * V + col < C) {
        float t = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) t += red[r][col];
        pm[(long)n * C + blockIdx.x * 32 * V + col] = t / (float)rows_per_clip;
    }
}

// logits[n][k] = b[k] + sum_c W[k][c] * pm[n][c]; one block per class k whose weight row stays in registers
// (up to 64 * FC_WREG input channels, more fall back to re-reading), one wavefront per clip at a time.
static constexpr int FC_WREG = 32;
__global__ void __launch_bounds__(256) fc_fwd_kernel(const float* __restrict__ pm, const float* __restrict__ W,
                                                     const float* __restrict__ b, float* __restrict__ logits, int N,
                                                     int C, int K) {
    const int k = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const float* w = W + (long)k * C;
    float wr[FC_WREG];
#pragma unroll
    for (int j = 0; j < FC_WREG; ++j) wr[j] = lane + 64 * j < C ? w[lane + 64 * j] : 0.f;
    const float bias = b[k];
    for (int n = threadIdx.x >> 6; n < N; n += 4) {
        const float* x = pm + (long)n * C;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int j = 0; j < FC_WREG; j += 2) {
            s0 = fmaf(wr[j], lane + 64 * j < C ? x[lane + 64 * j] : 0.f, s0);
            s1 = fmaf(wr[j + 1], lane + 64 * (j + 1) < C ? x[lane + 64 * (j + 1)] : 0.f, s1);
        }
        for (int c = lane + 64 * FC_WREG; c < C; c += 64) s0 = fmaf(w[c], x[c], s0);
        float s = s0 + s1;
        for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
        if (lane == 0) logits[(long)n * K + k] = s + bias;
    }
}

// One block of 16 wavefronts, one wavefront per clip at a time; loss = -mean_n log softmax(logits[n])[label[n]];
// dlogits = (softmax - onehot)/N.  The per-wavefront loss sums meet in LDS in a fixed order.
__global__ void __launch_bounds__(1024) softmax_ce_kernel(const float* __restrict__ logits, const int32_t* __restrict__ labels,
                                                          float* __restrict__ dlogits, float* __restrict__ loss, int N,
                                                          int K) {
    __shared__ float red[16];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float total = 0.f;
    for (int n = wv; n < N; n += 16) {
        const float* z = logits + (long)n * K;
        float mx = -3.0e38f;
        for (int k = lane; k < K; k += 64) mx = fmaxf(mx, z[k]);
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        float s = 0.f;
        for (int k = lane; k < K; k += 64) s += expf(z[k] - mx);
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        const float lse = mx + logf(s);
        int lab = labels[n];
        if (lab < 0 || lab >= K) lab = 0;   // out-of-range labels are treated as class 0
        for (int k = lane; k < K; k += 64)
            dlogits[(long)n * K + k] = (expf(z[k] - lse) - (k == lab ? 1.f : 0.f)) / (float)N;
        total += lse - z[lab];
    }
    if (lane == 0) red[wv] = total;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int i = 0; i < 16; ++i) t += red[i];
        *loss = t / (float)N;
    }
}

// dW[k][c] = sum_n dlogits[n][k]*pm[n][c]; db[k] = sum_n dlogits[n][k]
__global__ void __launch_bounds__(256) fc_bwd_w_kernel(const float* __restrict__ dlogits, const float* __restrict__ pm,
                                                       float* __restrict__ dW, float* __restrict__ db, int N, int C,
                                                       int K) {
    const int k = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < C) {
        float s = 0.f;
        for (int n = 0; n < N; ++n) s = fmaf(dlogits[(long)n * K + k], pm[(long)n * C + c], s);
        dW[(long)k * C + c] = s;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        float s = 0.f;
        for (int n = 0; n < N; ++n) s += dlogits[(long)n * K + k];
        db[k] = s;
    }
}

// dpm[n][c] = sum_k dlogits[n][k]*W[k][c]; block = 64 channels x 16 slices of the classes, eight clips per
// weight read; the slices meet in LDS in a fixed order.
__global__ void __launch_bounds__(1024) fc_bwd_x_kernel(const float* __restrict__ dlogits, const float* __restrict__ W,
                                                        float* __restrict__ dpm, int N, int C, int K) {
    __shared__ float red[16][8][64];
    const int n0 = blockIdx.y * 8;
    const int tx = threadIdx.x & 63, sl = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + tx;
    const float* dl[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) dl[j] = dlogits + (long)(n0 + j < N ? n0 + j : N - 1) * K;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    if (c < C) {
        for (int k = sl; k < K; k += 16) {
            const float w = W[(long)k * C + c];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = fmaf(dl[j][k], w, acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) red[sl][j][tx] = acc[j];
    __syncthreads();
    if (threadIdx.x < 512) {
        const int j = threadIdx.x >> 6;
        float t = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += red[q][j][tx];
        if (c < C && n0 + j < N) dpm[(long)(n0 + j) * C + c] = t;
    }
}

// dfeat[n][r][c] = dpm[n][c] / rows_per_clip; one 16-byte vector per thread (C is a multiple of the vector width)
template <typename T>
__global__ void __launch_bounds__(256) pool_mean_bwd_kernel(const float* __restrict__ dpm, T* __restrict__ dfeat,
                                                            int rows_per_clip, int C, long total_vec) {
    constexpr int V = Elem<T>::VEC;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total_vec) return;
    const int cv = C / V;
    const int c0 = (int)(i % cv) * V;
    const long n = i / ((long)rows_per_clip * cv);
    const float inv = 1.f / (float)rows_per_clip;
    Vec16<T> o;
#pragma unroll
    for (int j = 0; j < V; ++j) o.v[j] = Elem<T>::st(dpm[n * C + c0 + j] * inv);
    *(Vec16<T>*)(dfeat + i * V) = o;
}

// ---- bf16 working copies of all convolution weights, one launch per packing ---------------------
// Entry l packs params[in_off ..] = fp32 [Cout][Cin][taps] into out + out_off: forward order
// [Cout][taps][CinP] (channels >= Cin zero) or, with `flip`, the data-gradient order [Cin][flipped taps][Cout].
struct PackTable {
    int n;
    unsigned start[56];       // first output element of entry l in the launch's flat index space (start[n] = total)
    unsigned in_off[55];      // element offset into the fp32 parameter vector
    unsigned long long out_off[55];   // bf16 element offset from the output base (the workspace: 64 bits, it exceeds 8 GiB at a few dozen clips)
    unsigned short cout[55], cin[55], cinp[55], k[55];
    unsigned tstart[56];      // first 64 x 64 (Cout x Cin) tile of entry l, for pack_tiles_kernel; tiled == 0 if any
    int tiled;                // entry has a channel count that is not a multiple of 64 or padded input channels
};

__global__ void __launch_bounds__(256) pack_all_kernel(PackTable t, const float* __restrict__ params,
                                                       bf16_t* __restrict__ out, int flip) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= t.start[t.n]) return;
    int lo = 0, hi = t.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (t.start[mid] <= i) lo = mid; else hi = mid - 1;
    }
    const unsigned e = i - t.start[lo];
    const int Cout = t.cout[lo], Cin = t.cin[lo], CinP = t.cinp[lo], K = t.k[lo], taps = K * K;
    const float* w = params + t.in_off[lo];
    float v = 0.f;
    if (!flip) {          // e = (co * taps + tap) * CinP + ci
        const int ci = e % CinP, tap = (e / CinP) % taps, co = e / (CinP * taps);
        if (ci < Cin) v = w[((size_t)co * Cin + ci) * taps + tap];
    } else {              // e = (ci * taps + ftap) * Cout + co
        const int co = e % Cout, ftap = (e / Cout) % taps, ci = e / (Cout * taps);
        const int kw = K - 1 - ftap % K, kh = K - 1 - ftap / K;
        v = w[((size_t)co * Cin + ci) * taps + kh * K + kw];
    }
    out[(size_t)t.out_off[lo] + e] = f32_to_bf16(v);
}

// Same packings, both from one read of the fp32 weights, for tables whose channel counts are all multiples of 64:
// a block converts one 64 x 64 (Cout x Cin) tile of one convolution tap by tap; the forward order is written
// as read (input channels innermost), the data-gradient order (output channels innermost, taps flipped) goes
// through an LDS transpose.  `td` may equal `tf` when with_dgrad == 0.
__global__ void __launch_bounds__(256) pack_tiles_kernel(PackTable tf, PackTable td, const float* __restrict__ params,
                                                         bf16_t* __restrict__ out, int with_dgrad) {
    __shared__ bf16_t tile[64][66];
    const unsigned b = blockIdx.x;
    int lo = 0, hi = tf.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tf.tstart[mid] <= b) lo = mid; else hi = mid - 1;
    }
    const unsigned e = b - tf.tstart[lo];
    const int Cout = tf.cout[lo], Cin = tf.cin[lo], taps = tf.k[lo] * tf.k[lo];
    const int tiles_ci = Cin / 64;
    const int co0 = (int)(e / tiles_ci) * 64, ci0 = (int)(e % tiles_ci) * 64;
    const float* w = params + tf.in_off[lo];
    bf16_t* of = out + tf.out_off[lo];
    bf16_t* od = out + td.out_off[lo];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int tap = 0; tap < taps; ++tap) {
#pragma unroll 4
        for (int r = 0; r < 16; ++r) {
            const int co = r * 4 + ty;
            const bf16_t v = f32_to_bf16(w[((size_t)(co0 + co) * Cin + ci0 + tx) * taps + tap]);
            of[((size_t)(co0 + co) * taps + tap) * Cin + ci0 + tx] = v;
            if (with_dgrad) tile[co][tx] = v;
        }
        if (with_dgrad) {
            __syncthreads();
            const int ftap = taps - 1 - tap;
#pragma unroll 4
            for (int r = 0; r < 16; ++r) {
                const int ci = r * 4 + ty;
                od[((size_t)(ci0 + ci) * taps + ftap) * Cout + co0 + tx] = tile[tx][ci];
            }
            __syncthreads();
        }
    }
}

// ---- inference-mode BatchNorm parameters of the whole network in one launch ---------------------
// scale = gamma / sqrt(var + eps), shift = beta - mean * scale, written at the BatchNorm's position in the
// concatenated channel space (BatchNorms in parameter-table order).
struct BnTable {
    int n;
    unsigned start[56];       // first channel of BatchNorm l in the concatenated channel space (start[n] = total)
    unsigned g_off[55];       // element offsets of gamma / beta in the parameter vector
    unsigned b_off[55];
    unsigned s_off[55];       // offset of the BatchNorm's mean in the running-statistics vector (variance follows)
};

__global__ void __launch_bounds__(256) bn_eval_params_kernel(BnTable t, const float* __restrict__ params,
                                                             const float* __restrict__ bn_state, float eps,
                                                             float* __restrict__ scale, float* __restrict__ shift) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i >= t.start[t.n]) return;
    int lo = 0, hi = t.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (t.start[mid] <= i) lo = mid; else hi = mid - 1;
    }
    const unsigned c = i - t.start[lo], C = t.start[lo + 1] - t.start[lo];
    const float sc = params[t.g_off[lo] + c] / sqrtf(bn_state[t.s_off[lo] + C + c] + eps);
    scale[i] = sc;
    shift[i] = fmaf(-bn_state[t.s_off[lo] + c], sc, params[t.b_off[lo] + c]);
}

// ---- weight gradients of the several-tap convolutions: packed order [Cout][taps][Cin] -> [Cout][Cin][taps], all
// layers in one launch (the destination was zero-filled and nothing else writes it) ----------------------------
struct UnpackTable {
    int n;
    unsigned start[17];              // first (Cout, Cin) pair of entry l in the launch's flat index space (start[n] = total)
    unsigned src_off[16];            // float offset of the packed buffer from the base passed to the kernel
    unsigned dst_off[16];            // float offset into the gradient vector
    unsigned short cin[16], taps[16];
};

// One thread per (output channel, input channel) pair: its taps are read Cin floats apart (consecutive threads read
// consecutive addresses) and written as one contiguous run.
__global__ void __launch_bounds__(256) unpack_all_kernel(UnpackTable t, const float* __restrict__ packed,
                                                         float* __restrict__ grads) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;       // pair index in the launch's flat space
    if (i >= t.start[t.n]) return;
    int lo = 0, hi = t.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (t.start[mid] <= i) lo = mid; else hi = mid - 1;
    }
    const unsigned e = i - t.start[lo];                       // co * Cin + ci
    const unsigned taps = t.taps[lo], Cin = t.cin[lo];
    const unsigned ci = e % Cin, co = e / Cin;
    const float* src = packed + t.src_off[lo] + (size_t)co * taps * Cin + ci;
    float* dst = grads + t.dst_off[lo] + (size_t)e * taps;
    for (unsigned tap = 0; tap < taps; ++tap) dst[tap] = src[(size_t)tap * Cin];
}

// ---- SGD with momentum; weight decay only inside "decay" segments -----------------------------
struct SgdSegments {
    int n;
    unsigned start[120];     // ascending element offsets; segment s covers [start[s], start[s+1])
    unsigned char decays[120];
};

__device__ __forceinline__ int sgd_segment(const SgdSegments& seg, long i) {
    int lo = 0, hi = seg.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((long)seg.start[mid] <= i) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Four parameters per thread (16-byte accesses) where they lie in one segment, one at a time across a boundary.
__global__ void __launch_bounds__(256) sgd_kernel(float* __restrict__ w, float* __restrict__ v,
                                                  const float* __restrict__ g, long total, SgdSegments seg, float lr,
                                                  float momentum, float wd, float gscale) {
    const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= total) return;
    const int lo = sgd_segment(seg, i);
    if (i + 3 < total && (lo == seg.n - 1 || (long)seg.start[lo + 1] > i + 3)) {
        const float dec = seg.decays[lo] ? wd : 0.f;
        float4 wi = *(const float4*)(w + i), vi = *(const float4*)(v + i);
        const float4 gi = *(const float4*)(g + i);
        vi.x = fmaf(momentum, vi.x, gi.x * gscale + dec * wi.x);
        vi.y = fmaf(momentum, vi.y, gi.y * gscale + dec * wi.y);
        vi.z = fmaf(momentum, vi.z, gi.z * gscale + dec * wi.z);
        vi.w = fmaf(momentum, vi.w, gi.w * gscale + dec * wi.w);
        wi.x -= lr * vi.x; wi.y -= lr * vi.y; wi.z -= lr * vi.z; wi.w -= lr * vi.w;
        *(float4*)(v + i) = vi;
        *(float4*)(w + i) = wi;
        return;
    }
    for (long e = i; e < i + 4 && e < total; ++e) {
        const float we = w[e];
        const float ge = g[e] * gscale + (seg.decays[sgd_segment(seg, e)] ? wd * we : 0.f);
        const float ve = fmaf(momentum, v[e], ge);
        v[e] = ve;
        w[e] = we - lr * ve;
    }
}

// Gradient accumulation over micro-batches: acc = g (first micro-batch) or acc += g.
__global__ void __launch_bounds__(256) grad_accum_kernel(float* __restrict__ acc, const float* __restrict__ g, long n,
                                                         int first) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    acc[i] = first ? g[i] : acc[i] + g[i];
}

// micro-batch `index` of `count` whose gradients are summed in `buf` (fp32 [param_count])
struct GradAccum {
    float* buf;
    int index, count;
};

// ---- the step ---------------------------------------------------------------------------------
#define RUN(expr)                          \
    do {                                   \
        if (!dry) TSM_TRY(expr);           \
    } while (0)
#define LAUNCH_CHECK(what) RUN(check_launch(what))

// Question to the step's workspace plan: where does the named forward activation live (see
// tsm_resnet50_workspace_tensor)?  Answered by a dry pass of the plan over a placeholder base address.
struct WsQuery {
    const char* name;
    size_t offset;
    int shape[4];
    int elem_bytes;
    bool found;
};
static char* const kQueryBase = (char*)(uintptr_t)(1u << 20);   // never dereferenced

static int r50_step(const tsm_r50_desc* d, const void* clips, const int32_t* labels, float* params, float* momentum,
                    float* bn_state, float* grads_out, float* loss_out, float* logits_out, int update, void* wsp,
                    size_t ws_bytes, bool dry, hipStream_t s, size_t* need, const GradAccum* acc = nullptr,
                    WsQuery* query = nullptr) {
    const char* who = query ? "tsm_resnet50_workspace_tensor" : acc ? "tsm_resnet50_accum_step" : "tsm_resnet50_step";
    if (!d) return fail(TSM_ERR_NULLPTR, "%s: null descriptor", who);
    if (d->N <= 0 || d->T <= 0 || d->size < 32 || d->num_classes <= 0)
        return fail(TSM_ERR_SHAPE, "%s: N, T, num_classes must be positive and size >= 32", who);
    if (d->size % 32) return fail(TSM_ERR_SHAPE, "%s: size must be a multiple of 32", who);
    if ((long)d->N * d->T > 65535) return fail(TSM_ERR_SHAPE, "%s: too many frames", who);
    if (d->dtype != TSM_F32 && d->dtype != TSM_BF16) return fail(TSM_ERR_DTYPE, "%s: unknown dtype %d", who, d->dtype);
    int fold_chk = 0;
    if (fold_of(64, d->fold_div, &fold_chk) != TSM_OK) return fail(TSM_ERR_FOLD, "%s: invalid fold_div %d", who, d->fold_div);
    if (!dry) {
        if (!clips || !labels || !params || !momentum || !loss_out) return fail(TSM_ERR_NULLPTR, "%s: null pointer", who);
        if (!aligned16(clips) || !aligned16(params) || !aligned16(momentum) || !aligned16(wsp) || !aligned16(grads_out))
            return fail(TSM_ERR_ALIGN, "%s: pointers must be 16-byte aligned", who);
        size_t req = 0;
        TSM_TRY(r50_step(d, clips, labels, params, momentum, bn_state, grads_out, loss_out, logits_out, update, nullptr,
                         0, true, s, &req));
        if (req > ws_bytes) return fail(TSM_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu", who, ws_bytes, req);
        if (!wsp) return fail(TSM_ERR_NULLPTR, "%s: null workspace", who);
    }
    static thread_local std::vector<TensorInfo> table;
    static thread_local int table_classes = -1;
    if (table_classes != d->num_classes) {
        table = build_table(d->num_classes);
        table_classes = d->num_classes;
    }
    const int64_t nparams = table.back().offset + table.back().count();
    const int F = d->N * d->T, T = d->T, S = d->size, K = d->num_classes;
    const int dtype = d->dtype;
    const bool bf = dtype == TSM_BF16;
    const size_t es = dtype_size(dtype);
    const int VEC = bf ? 8 : 4;
    Arena A(dry ? (query ? (void*)kQueryBase : nullptr) : wsp, (size_t)-1);

    // running-statistics slots follow the BatchNorm order of the table
    int64_t bn_off = 0;
    auto run_slot = [&](int C, float** rm, float** rv) {
        if (bn_state) {
            *rm = bn_state + bn_off;
            *rv = bn_state + bn_off + C;
        } else {
            *rm = *rv = nullptr;
        }
        bn_off += 2 * C;
    };

    // (reserved whether or not the caller passes grads_out / logits_out: the layout of the workspace must not depend
    // on the optional outputs, tsm_resnet50_workspace_tensor describes it from the descriptor alone)
    float* const grads_ws = A.take_n<float>((size_t)nparams);
    float* grads = grads_out ? grads_out : grads_ws;

    auto P = [&](const std::string& name) { return params + table[find_tensor(table, name)].offset; };
    auto G = [&](const std::string& name) { return grads + table[find_tensor(table, name)].offset; };
    // bf16: working copies of the convolution weights in both packings; fp32: the master weights are used directly
    PackTable pk_fwd, pk_dg;
    pk_fwd.n = pk_dg.n = 0;
    pk_fwd.start[0] = pk_dg.start[0] = 0;
    pk_fwd.tstart[0] = pk_dg.tstart[0] = 0;
    pk_fwd.tiled = pk_dg.tiled = 1;
    bf16_t* const pack_base = (bf16_t*)(dry ? nullptr : wsp);   // packed buffers are addressed relative to the workspace
    auto pack_entry = [&](PackTable& t, const std::string& name, int Cout, int Cin, int k, int CinP, size_t count,
                          const bf16_t* dst) {
        const int l = t.n++;
        t.in_off[l] = (unsigned)table[find_tensor(table, name)].offset;
        t.out_off[l] = (unsigned long long)(dst - pack_base);
        t.cout[l] = (unsigned short)Cout; t.cin[l] = (unsigned short)Cin; t.cinp[l] = (unsigned short)CinP;
        t.k[l] = (unsigned short)k;
        t.start[l + 1] = t.start[l] + (unsigned)count;
        t.tstart[l + 1] = t.tstart[l] + (unsigned)((Cout / 64) * (Cin / 64));
        if (Cout % 64 || Cin % 64 || CinP != Cin) t.tiled = 0;
    };
    auto pack_conv = [&](const std::string& name, int Cout, int Cin, int k, int CinP, const bf16_t** wp,
                         const bf16_t** wd) -> int {
        *wp = nullptr;
        if (wd) *wd = nullptr;
        if (!bf) return TSM_OK;
        if (pk_fwd.n >= 55 || pk_dg.n >= 55) return fail(TSM_ERR_UNSUPPORTED, "%s: too many convolutions", who);
        const size_t nf = (size_t)Cout * CinP * k * k;
        bf16_t* a = A.take_n<bf16_t>(nf);
        pack_entry(pk_fwd, name, Cout, Cin, k, CinP, nf, a);
        *wp = a;
        if (wd) {
            const size_t nd = (size_t)Cout * Cin * k * k;
            bf16_t* b2 = A.take_n<bf16_t>(nd);
            pack_entry(pk_dg, name, Cout, Cin, k, Cin, nd, b2);
            *wd = b2;
        }
        return TSM_OK;
    };

    size_t scratch_need = 0;

    // ---- stem: bf16 runs it in space-to-depth form (see clips_to_s2d_kernel); fp32 keeps the three channels
    const int H1 = S / 2, Hp = S / 4;     // conv1 output, pooled output
    const int Hs = H1 + 3;                // space-to-depth image, with halo
    bf16_t* wp0 = bf ? A.take_n<bf16_t>(64 * 256) : nullptr;
    void* x0 = bf ? A.take((size_t)F * Hs * Hs * 16 * es) : A.take((size_t)F * S * S * 3 * es);
    void* y0 = A.take((size_t)F * H1 * H1 * 64 * es);
    BnVec bn0;
    bn0.mean = A.take_n<float>(64); bn0.rstd = A.take_n<float>(64); bn0.scale = A.take_n<float>(64); bn0.shift = A.take_n<float>(64);
    uint8_t* arg0 = A.take_n<uint8_t>((size_t)F * Hp * Hp * 64);
    void* p0 = A.take((size_t)F * Hp * Hp * 64 * es);
    ConvP stem{};
    stem.F = F; stem.T = T; stem.Ho = H1; stem.Wo = H1; stem.Cout = 64; stem.KT = 1; stem.fold = 0;
    if (bf) {
        stem.H = Hs; stem.W = Hs; stem.Cin = 64; stem.pitch = 16; stem.KH = 4; stem.KW = 1; stem.stride = 1; stem.pad = 0;
    } else {
        stem.H = S; stem.W = S; stem.Cin = 3; stem.KH = 7; stem.KW = 7; stem.stride = 2; stem.pad = 3;
    }
    float *rm0, *rv0;
    run_slot(64, &rm0, &rv0);
    const int nb0f = bf ? conv_mfma_fwd_blocks(stem) : red_blocks(stem.rows_out(), 64, dtype);
    // blocks of the stem backward kernel (rows of its partial buffer): 32 or 16 pixels per block step, a few
    // steps per block
    const int nb0b = (int)std::min<long>(4096, std::max<long>(1, stem.rows_out() / 128));
    float* part0 = A.take_n<float>((size_t)(nb0f > nb0b ? nb0f : nb0b) * 128);
    float* coef0 = A.take_n<float>(3 * 64);
    float* dwp0 = A.take_n<float>((size_t)64 * 256);

    // ---- blocks: plans, saved buffers, outputs
    struct Blk {
        BlockPlan plan;
        void* out;
        const void* in;
    };
    std::vector<Blk> blks;
    {
        int cin = 64, h = Hp;
        const void* cur = p0;
        for (const StageSpec& st : kStages) {
            for (int b = 0; b < st.blocks; ++b) {
                const std::string pre = std::string(st.name) + "." + std::to_string(b) + ".";
                tsm_block_desc bd{};
                bd.kind = TSM_BLOCK_BOTTLENECK; bd.N = d->N; bd.T = T; bd.Cin = cin; bd.H = h; bd.W = h;
                bd.Cmid = st.mid; bd.Cout = 4 * st.mid; bd.stride = b == 0 ? st.stride : 1; bd.has_projection = b == 0;
                bd.fold_div = d->fold_div; bd.dtype = dtype; bd.layout = TSM_NTHWC; bd.bn_eps = d->bn_eps;
                Blk blk;
                TSM_TRY(make_block_plan(&bd, &blk.plan, who));
                BlockPlan& pl = blk.plan;
                pl.bn_momentum = d->bn_momentum;
                pl.grads_prezeroed = true;
                const char* cn[3] = {"c1.w", "c2.w", "c3.w"};
                const char* bnn[3] = {"bn1", "bn2", "bn3"};
                for (int i = 0; i < 3; ++i) {
                    StageDef& sd = pl.st[i];
                    TSM_TRY(pack_conv(pre + cn[i], sd.p.Cout, sd.p.Cin, sd.p.KH, sd.p.Cin, &sd.wp, &sd.wd));
                    sd.w = P(pre + cn[i]);   // fp32 master weights: read by the fp32 kernels only
                    sd.g = P(pre + bnn[i] + ".g"); sd.b = P(pre + bnn[i] + ".b");
                    sd.dw = G(pre + cn[i]); sd.dg = G(pre + bnn[i] + ".g"); sd.db = G(pre + bnn[i] + ".b");
                    run_slot(sd.p.Cout, &sd.run_mean, &sd.run_var);
                }
                if (pl.proj) {
                    StageDef& sd = pl.ds;
                    TSM_TRY(pack_conv(pre + "ds.w", sd.p.Cout, sd.p.Cin, 1, sd.p.Cin, &sd.wp, &sd.wd));
                    sd.w = P(pre + "ds.w");
                    sd.g = P(pre + "dsbn.g"); sd.b = P(pre + "dsbn.b");
                    sd.dw = G(pre + "ds.w"); sd.dg = G(pre + "dsbn.g"); sd.db = G(pre + "dsbn.b");
                    run_slot(sd.p.Cout, &sd.run_mean, &sd.run_var);
                }
                block_saved_layout(pl, A, false);
                const ConvP& last = pl.st[2].p;
                blk.out = A.take((size_t)last.rows_out() * last.Cout * es);
                // the output's ReLU decisions as bits: what the next block's first data gradient reads as its mask
                pl.out_bits = block_tail_writes_bits(dtype, last.Cout)
                                  ? A.take_n<uint8_t>((size_t)last.rows_out() * last.Cout / 8) : nullptr;
                blk.in = cur;
                cur = blk.out;
                blks.push_back(blk);
                cin = 4 * st.mid;
                h = last.Ho;
            }
        }
    }
    // several-tap convolutions on the MFMA path accumulate their weight gradient in the packed order: one
    // contiguous region, zeroed with one fill and permuted into the gradient vector with one launch
    UnpackTable unp;
    unp.n = 0;
    unp.start[0] = 0;
    float* const dwp_base = (float*)(dry ? nullptr : (char*)wsp + A.used);
    size_t dwp_bytes = 0;
    if (bf) {
        const size_t used0 = A.used;
        for (Blk& blk : blks) {
            for (int i = 0; i < 3; ++i) {
                StageDef& sd = blk.plan.st[i];
                if (sd.p.taps() <= 1 || !mfma_conv_supported(sd.p) || unp.n >= 16) continue;
                const size_t n = (size_t)sd.p.Cout * sd.p.K();
                sd.dwp = A.take_n<float>(n);
                const int l = unp.n++;
                unp.src_off[l] = (unsigned)(sd.dwp - dwp_base);
                unp.dst_off[l] = (unsigned)(sd.dw - grads);
                unp.cin[l] = (unsigned short)sd.p.Cin;
                unp.taps[l] = (unsigned short)sd.p.taps();
                unp.start[l + 1] = unp.start[l] + (unsigned)(n / sd.p.taps());
            }
        }
        dwp_bytes = A.used - used0;
    }
    const ConvP& lastp = blks.back().plan.st[2].p;
    const int Cf = lastp.Cout, rows_clip = T * lastp.Ho * lastp.Wo;
    float* pm = A.take_n<float>((size_t)d->N * Cf);
    float* dpm = A.take_n<float>((size_t)d->N * Cf);
    float* const logits_ws = A.take_n<float>((size_t)d->N * K);
    float* logits = logits_out ? logits_out : logits_ws;
    float* dlogits = A.take_n<float>((size_t)d->N * K);
    // gradient ping-pong buffers: the largest activation between blocks
    size_t act_max = (size_t)F * Hp * Hp * 64 * es;
    for (const Blk& b : blks) {
        const ConvP& l = b.plan.st[2].p;
        const size_t by = (size_t)l.rows_out() * l.Cout * es;
        if (by > act_max) act_max = by;
    }
    void* dbuf[2] = {A.take(act_max), A.take(act_max)};
    // Chaining: the data gradient that produces block i's input gradient also applies block i-1's output
    // ReLU mask and accumulates the sums of its last BatchNorm, when block i-1 has an identity shortcut and the
    // kernel can fuse.
    std::vector<float*> chain_part(blks.size(), nullptr);
    std::vector<int> chain_nb(blks.size(), 0);
    for (size_t i = 1; i < blks.size(); ++i) {
        if (blks[i - 1].plan.proj) continue;
        const int nbf = conv_dgrad_fuse_blocks(blks[i].plan.st[0].p, dtype);
        if (!nbf) continue;
        chain_nb[i - 1] = nbf;
        chain_part[i - 1] = A.take_n<float>((size_t)nbf * 2 * blks[i - 1].plan.st[2].p.Cout);
    }
    void* da0 = A.take((size_t)F * H1 * H1 * 64 * es);
    if (query) {
        // forward activations a step leaves behind in its workspace (nothing in the backward pass writes them)
        auto answer = [&](const void* p, int f, int h, int w, int c, int eb) {
            query->offset = (size_t)((const char*)p - kQueryBase);
            query->shape[0] = f; query->shape[1] = h; query->shape[2] = w; query->shape[3] = c;
            query->elem_bytes = eb;
            query->found = true;
        };
        const std::string q = query->name;
        if (q == "stem.y") answer(y0, F, H1, H1, 64, (int)es);
        else if (q == "stem.bn_scale") answer(bn0.scale, 64, 1, 1, 1, 4);
        else if (q == "stem.bn_shift") answer(bn0.shift, 64, 1, 1, 1, 4);
        else if (q == "stem.pool_arg") answer(arg0, F, Hp, Hp, 64, 1);
        else if (q == "stem.pool") answer(p0, F, Hp, Hp, 64, (int)es);
        else {
            size_t bi = 0;
            for (const StageSpec& st : kStages) {
                for (int b = 0; b < st.blocks; ++b, ++bi) {
                    const std::string pre = std::string(st.name) + "." + std::to_string(b) + ".";
                    if (q.compare(0, pre.size(), pre) != 0) continue;
                    const BlockPlan& pl = blks[bi].plan;
                    const std::string t = q.substr(pre.size());
                    const ConvP &p1 = pl.st[0].p, &p2 = pl.st[1].p, &p3 = pl.st[2].p;
                    if (t == "y1") answer(pl.y[0], F, p1.Ho, p1.Wo, p1.Cout, (int)es);
                    else if (t == "z1") answer(pl.z[0], F, p1.Ho, p1.Wo, p1.Cout, (int)es);
                    else if (t == "y2") answer(pl.y[1], F, p2.Ho, p2.Wo, p2.Cout, (int)es);
                    else if (t == "z2") answer(pl.z[1], F, p2.Ho, p2.Wo, p2.Cout, (int)es);
                    else if (t == "y3") answer(pl.y[2], F, p3.Ho, p3.Wo, p3.Cout, (int)es);
                    else if (t == "out") answer(blks[bi].out, F, p3.Ho, p3.Wo, p3.Cout, (int)es);
                    else if (t == "yd" && pl.proj) answer(pl.yd, F, p3.Ho, p3.Wo, p3.Cout, (int)es);
                }
            }
        }
        return TSM_OK;
    }
    char* scratch_base = dry ? nullptr : (char*)wsp + A.used;
    const size_t scratch_cap = dry ? (size_t)-1 : (ws_bytes > A.used ? ws_bytes - A.used : 0);
    auto note = [&](const Arena& sc) { if (sc.used > scratch_need) scratch_need = sc.used; };

    // The fills and the weight packing are needed from the first residual block on: they run on the second stream
    // beside the stem and are joined in front of the blocks (on every path out of this function).
    struct Branch {
        hipStream_t s, b;
        bool open;
        int end() { const int rc = open ? side_branch_end(s, b) : TSM_OK; open = false; return rc; }
        ~Branch() { (void)end(); }
    } prep{s, dry ? s : side_branch_begin(s), !dry};
    const hipStream_t sp = prep.b;
    // every weight gradient is accumulated with atomics: one fill for the whole gradient vector
    RUN(fill_zero(grads, (size_t)nparams * sizeof(float), sp));
    if (dwp_bytes) RUN(fill_zero(dwp_base, dwp_bytes, sp));
    if (bf && !dry) {   // bf16 working copies of all convolution weights in both packings
        if (pk_fwd.tiled && pk_dg.tiled && pk_fwd.n == pk_dg.n) {
            pack_tiles_kernel<<<dim3(pk_fwd.tstart[pk_fwd.n]), dim3(256), 0, sp>>>(pk_fwd, pk_dg, params, pack_base, 1);
            LAUNCH_CHECK("pack_weights");
        } else {
            pack_all_kernel<<<dim3(cdiv(pk_fwd.start[pk_fwd.n], 256)), dim3(256), 0, sp>>>(pk_fwd, params, pack_base, 0);
            LAUNCH_CHECK("pack_weights_fwd");
            pack_all_kernel<<<dim3(cdiv(pk_dg.start[pk_dg.n], 256)), dim3(256), 0, sp>>>(pk_dg, params, pack_base, 1);
            LAUNCH_CHECK("pack_weights_dgrad");
        }
    }

    // ================= forward =================
    {
        if (bf) {
            if (!dry) {
                const long total = (long)F * Hs * Hs;
                clips_to_s2d_kernel<<<dim3(cdiv(total, 256)), dim3(256), 0, s>>>((const bf16_t*)clips, (uint4*)x0, S, Hs, total);
                LAUNCH_CHECK("clips_to_s2d");
                stem_pack_kernel<<<dim3(64), dim3(256), 0, s>>>(P("conv1.w"), wp0);
                LAUNCH_CHECK("stem_pack");
            }
        } else {
            RUN(transpose_frames(clips, x0, F, 3, S * S, 4, s));
        }
        if (bf) {
            RUN(conv_mfma_fwd(stem, (const bf16_t*)x0, wp0, (bf16_t*)y0, part0, nullptr, s));
        } else {
            RUN(conv_direct_fwd(stem, dtype, x0, P("conv1.w"), y0, s));
            RUN(channel_stats(dtype, y0, stem.rows_out(), 64, part0, s));
        }
        RUN(bn_finalize(part0, nb0f, stem.rows_out(), 64, P("bn1.g"), P("bn1.b"), d->bn_eps, bn0, rm0, rv0,
                        d->bn_momentum, s));
        const int cv = 64 / VEC;
        const long ptotal = (long)F * Hp * Hp * cv;
        if (!dry) {
            if (bf)
                stem_pool_fwd_kernel<bf16_t><<<dim3(cdiv(ptotal, 256)), dim3(256), 0, s>>>((const bf16_t*)y0, bn0.scale, bn0.shift, (bf16_t*)p0, arg0, H1, H1, Hp, Hp, cv, ptotal);
            else
                stem_pool_fwd_kernel<float><<<dim3(cdiv(ptotal, 256)), dim3(256), 0, s>>>((const float*)y0, bn0.scale, bn0.shift, (float*)p0, arg0, H1, H1, Hp, Hp, cv, ptotal);
            LAUNCH_CHECK("stem_pool_fwd");
        }
    }
    TSM_TRY(prep.end());
    for (Blk& b : blks) {
        Arena sc(scratch_base, scratch_cap);
        TSM_TRY(block_fwd_impl(b.plan, b.in, b.out, sc, dry, s));
        note(sc);
    }
    if (!dry) {
        if (bf)
            pool_mean_kernel<bf16_t><<<dim3(cdiv(Cf, 256), d->N), dim3(256), 0, s>>>((const bf16_t*)blks.back().out, pm, rows_clip, Cf);
        else
            pool_mean_kernel<float><<<dim3(cdiv(Cf, 128), d->N), dim3(256), 0, s>>>((const float*)blks.back().out, pm, rows_clip, Cf);
        LAUNCH_CHECK("pool_mean");
        fc_fwd_kernel<<<dim3(K), dim3(256), 0, s>>>(pm, P("fc.w"), P("fc.b"), logits, d->N, Cf, K);
        LAUNCH_CHECK("fc_fwd");
        softmax_ce_kernel<<<dim3(1), dim3(1024), 0, s>>>(logits, labels, dlogits, loss_out, d->N, K);
        LAUNCH_CHECK("softmax_ce");
        // ================= backward =================
        fc_bwd_w_kernel<<<dim3(cdiv(Cf, 256), K), dim3(256), 0, s>>>(dlogits, pm, G("fc.w"), G("fc.b"), d->N, Cf, K);
        LAUNCH_CHECK("fc_bwd_w");
        fc_bwd_x_kernel<<<dim3(cdiv(Cf, 64), cdiv(d->N, 8)), dim3(1024), 0, s>>>(dlogits, P("fc.w"), dpm, d->N, Cf, K);
        LAUNCH_CHECK("fc_bwd_x");
        const long ftotal = (long)d->N * rows_clip * Cf;
        if (bf)
            pool_mean_bwd_kernel<bf16_t><<<dim3(cdiv(ftotal / 8, 256)), dim3(256), 0, s>>>(dpm, (bf16_t*)dbuf[0], rows_clip, Cf, ftotal / 8);
        else
            pool_mean_bwd_kernel<float><<<dim3(cdiv(ftotal / 4, 256)), dim3(256), 0, s>>>(dpm, (float*)dbuf[0], rows_clip, Cf, ftotal / 4);
        LAUNCH_CHECK("pool_mean_bwd");
    }
    // The blocks' scratch alternates between two halves of the scratch region, so that the weight gradients of a
    // block, which run on the library's second stream, need not be complete before the next block starts (see
    // block_bwd_impl); whatever path leaves this function first takes the joins still open.
    struct Flush {
        hipStream_t s; bool on;
        ~Flush() { if (on) (void)block_bwd_flush(s); }
    } flush{s, !dry};
    const size_t half_cap = dry ? (size_t)-1 : (scratch_cap / 2) & ~(size_t)255;
    size_t bwd_need = 0;
    int cur = 0;
    for (int i = (int)blks.size() - 1; i >= 0; --i) {
        Blk& b = blks[i];
        Arena sc(dry ? nullptr : scratch_base + (size_t)(i & 1) * half_cap, half_cap);
        DgradFuse fz;
        b.plan.dx_fuse = nullptr;
        if (i > 0 && chain_nb[i - 1]) {
            BlockPlan& pp = blks[i - 1].plan;
            fz = DgradFuse{(const bf16_t*)blks[i - 1].out, (const bf16_t*)pp.y[2], pp.bn[2].mean, pp.bn[2].rstd, chain_part[i - 1], pp.out_bits};
            b.plan.dx_fuse = &fz;
            pp.dout_part = dry ? (const float*)1 : chain_part[i - 1];   // (dry run: only the flag matters)
            pp.dout_nb = chain_nb[i - 1];
        } else if (i > 0 && blks[i - 1].plan.proj && conv_dgrad_fuse_blocks(b.plan.st[0].p, dtype)) {
            // block i-1 has a projection shortcut (two BatchNorms share its output gradient): the data gradient
            // applies its output ReLU mask only, the two pairs of sums are reduced from the masked gradient
            fz = DgradFuse{(const bf16_t*)blks[i - 1].out, nullptr, nullptr, nullptr, nullptr, blks[i - 1].plan.out_bits};
            b.plan.dx_fuse = &fz;
            blks[i - 1].plan.dout_masked = true;
        }
        TSM_TRY(block_bwd_impl(b.plan, b.in, b.out, dbuf[cur], dbuf[cur ^ 1], sc, dry, s, i & 1));
        if (sc.used > bwd_need) bwd_need = sc.used;
        cur ^= 1;
    }
    if (!dry) TSM_TRY(block_bwd_flush(s));
    if (2 * ((bwd_need + 255) & ~(size_t)255) > scratch_need) scratch_need = 2 * ((bwd_need + 255) & ~(size_t)255);
    {   // stem backward: max-pool routing + ReLU mask, BatchNorm backward, weight gradient (no input gradient)
        const long rows0 = stem.rows_out();
        if (!dry) {
            const dim3 blk(64 / VEC, 256 / (64 / VEC));
            if (bf && H1 % 2 == 0)
                stem_pool_bwd_patch_kernel<bf16_t><<<dim3(nb0b), blk, 0, s>>>((const bf16_t*)dbuf[cur], arg0, (const bf16_t*)y0, bn0.scale, bn0.shift, bn0.mean, bn0.rstd, (bf16_t*)da0, part0, H1, H1, Hp, Hp, rows0 / 4);
            else if (bf)
                stem_pool_bwd_kernel<bf16_t><<<dim3(nb0b), blk, 0, s>>>((const bf16_t*)dbuf[cur], arg0, (const bf16_t*)y0, bn0.scale, bn0.shift, bn0.mean, bn0.rstd, (bf16_t*)da0, part0, H1, H1, Hp, Hp, rows0);
            else
                stem_pool_bwd_kernel<float><<<dim3(nb0b), blk, 0, s>>>((const float*)dbuf[cur], arg0, (const float*)y0, bn0.scale, bn0.shift, bn0.mean, bn0.rstd, (float*)da0, part0, H1, H1, Hp, Hp, rows0);
            LAUNCH_CHECK("stem_pool_bwd");
        }
        RUN(bn_bwd_coeffs(part0, nb0b, rows0, 64, bn0.mean, bn0.rstd, P("bn1.g"), coef0, G("bn1.g"), G("bn1.b"), s));
        // nothing but the weight gradient reads the stem's dy: on the bf16 path its loader forms it from dz and y0
        const bool affine = bf && conv_mfma_wgrad_affine_ok(stem);
        if (!affine) RUN(bn_bwd_apply(dtype, da0, y0, stem.rows_out(), 64, coef0, da0, s));
        // the gradient buffer was zeroed at the start of the step; both kernels add into it
        if (bf) {
            RUN(fill_zero(dwp0, (size_t)64 * 256 * sizeof(float), s));
            RUN(conv_mfma_wgrad(stem, (const bf16_t*)x0, (const bf16_t*)da0, dwp0, 64, true, s,
                                affine ? (const bf16_t*)y0 : nullptr, affine ? coef0 : nullptr));
            if (!dry) {
                stem_unpack_kernel<<<dim3(64), dim3(256), 0, s>>>(dwp0, G("conv1.w"));
                LAUNCH_CHECK("stem_unpack");
            }
        } else
            RUN(conv_direct_wgrad(stem, dtype, x0, da0, G("conv1.w"), s));
    }
    if (unp.n && !dry) {
        unpack_all_kernel<<<dim3(cdiv(unp.start[unp.n], 256)), dim3(256), 0, s>>>(unp, dwp_base, grads);
        LAUNCH_CHECK("unpack_wgrad");
    }
    // ================= update =================
    if (acc && !dry) {
        grad_accum_kernel<<<dim3(cdiv(nparams, 256)), dim3(256), 0, s>>>(acc->buf, grads, nparams, acc->index == 0);
        LAUNCH_CHECK("grad_accum");
    }
    if (update && !dry) {
        SgdSegments seg;
        seg.n = 0;
        for (const TensorInfo& ti : table) {
            if (seg.n == 0 || (bool)seg.decays[seg.n - 1] != ti.decays) {
                if (seg.n >= 120) return fail(TSM_ERR_UNSUPPORTED, "%s: too many optimiser segments", who);
                seg.start[seg.n] = (unsigned)ti.offset;
                seg.decays[seg.n] = ti.decays ? 1 : 0;
                ++seg.n;
            }
        }
        const float* gsrc = acc ? acc->buf : grads;
        sgd_kernel<<<dim3(cdiv(nparams, 1024)), dim3(256), 0, s>>>(params, momentum, gsrc, nparams, seg, d->lr, d->momentum,
                                                                  d->weight_decay, acc ? 1.f / (float)acc->count : 1.f);
        LAUNCH_CHECK("sgd");
    }
    if (need) *need = A.used + scratch_need;
    return TSM_OK;
}

}  // namespace tsm

using namespace tsm;

// ---- forward only (inference): BatchNorm with the running statistics, folded into the convolution
// epilogues on the bf16 path; nothing is saved for a backward pass ------------------------------------
static int r50_infer(const tsm_r50_desc* d, const void* clips, const float* params, const float* bn_state,
                     float* logits_out, void* wsp, size_t ws_bytes, bool dry, hipStream_t s, size_t* need) {
    const char* who = "tsm_resnet50_infer";
    if (!d) return fail(TSM_ERR_NULLPTR, "%s: null descriptor", who);
    if (d->N <= 0 || d->T <= 0 || d->size < 32 || d->num_classes <= 0)
        return fail(TSM_ERR_SHAPE, "%s: N, T, num_classes must be positive and size >= 32", who);
    if (d->size % 32) return fail(TSM_ERR_SHAPE, "%s: size must be a multiple of 32", who);
    if ((long)d->N * d->T > 65535) return fail(TSM_ERR_SHAPE, "%s: too many frames", who);
    if (d->dtype != TSM_F32 && d->dtype != TSM_BF16) return fail(TSM_ERR_DTYPE, "%s: unknown dtype %d", who, d->dtype);
    int fold_chk = 0;
    if (fold_of(64, d->fold_div, &fold_chk) != TSM_OK) return fail(TSM_ERR_FOLD, "%s: invalid fold_div %d", who, d->fold_div);
    if (!(d->bn_eps >= 0.f)) return fail(TSM_ERR_SHAPE, "%s: bn_eps must be >= 0", who);
    if (!dry) {
        if (!clips || !params || !bn_state || !logits_out) return fail(TSM_ERR_NULLPTR, "%s: null pointer", who);
        if (!aligned16(clips) || !aligned16(params) || !aligned16(wsp))
            return fail(TSM_ERR_ALIGN, "%s: pointers must be 16-byte aligned", who);
        size_t req = 0;
        TSM_TRY(r50_infer(d, clips, params, bn_state, logits_out, nullptr, 0, true, s, &req));
        if (req > ws_bytes) return fail(TSM_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu", who, ws_bytes, req);
        if (!wsp) return fail(TSM_ERR_NULLPTR, "%s: null workspace", who);
    }
    static thread_local std::vector<TensorInfo> table;
    static thread_local int table_classes = -1;
    if (table_classes != d->num_classes) {
        table = build_table(d->num_classes);
        table_classes = d->num_classes;
    }
    const int F = d->N * d->T, T = d->T, S = d->size, K = d->num_classes;
    const int dtype = d->dtype;
    const bool bf = dtype == TSM_BF16;
    const size_t es = dtype_size(dtype);
    const int VEC = bf ? 8 : 4;
    Arena A(dry ? nullptr : wsp, (size_t)-1);
    auto P = [&](const std::string& name) { return params + table[find_tensor(table, name)].offset; };

    // ---- BatchNorm parameters: one launch over all channels
    BnTable bt;
    bt.n = 0;
    bt.start[0] = 0;
    unsigned s_off = 0;
    for (size_t i = 0; i < table.size(); ++i) {
        const std::string& nm = table[i].name;
        if (nm.size() < 2 || nm.compare(nm.size() - 2, 2, ".g") != 0) continue;
        if (bt.n >= 55) return fail(TSM_ERR_UNSUPPORTED, "%s: too many BatchNorms", who);
        const unsigned C = (unsigned)table[i].count();
        bt.g_off[bt.n] = (unsigned)table[i].offset;
        bt.b_off[bt.n] = (unsigned)table[i + 1].offset;   // beta follows gamma in the table
        bt.s_off[bt.n] = s_off;
        bt.start[bt.n + 1] = bt.start[bt.n] + C;
        s_off += 2 * C;
        ++bt.n;
    }
    const unsigned nch = bt.start[bt.n];
    float* scale_all = A.take_n<float>(nch);
    float* shift_all = A.take_n<float>(nch);
    int bn_next = 0;   // BatchNorms are consumed in table order
    auto bn_slot = [&](const float** sc, const float** sh) {
        *sc = scale_all + bt.start[bn_next];
        *sh = shift_all + bt.start[bn_next];
        ++bn_next;
    };

    // ---- forward weights (bf16: packed working copies, one launch)
    PackTable pk;
    pk.n = 0;
    pk.start[0] = 0;
    pk.tstart[0] = 0;
    pk.tiled = 1;
    bf16_t* const pack_base = (bf16_t*)(dry ? nullptr : wsp);
    auto pack_conv = [&](const std::string& name, int Cout, int Cin, int k, const bf16_t** wp) -> int {
        *wp = nullptr;
        if (!bf) return TSM_OK;
        if (pk.n >= 55) return fail(TSM_ERR_UNSUPPORTED, "%s: too many convolutions", who);
        const size_t nf = (size_t)Cout * Cin * k * k;
        bf16_t* a = A.take_n<bf16_t>(nf);
        const int l = pk.n++;
        pk.in_off[l] = (unsigned)table[find_tensor(table, name)].offset;
        pk.out_off[l] = (unsigned long long)(a - pack_base);
        pk.cout[l] = (unsigned short)Cout; pk.cin[l] = (unsigned short)Cin; pk.cinp[l] = (unsigned short)Cin;
        pk.k[l] = (unsigned short)k;
        pk.start[l + 1] = pk.start[l] + (unsigned)nf;
        pk.tstart[l + 1] = pk.tstart[l] + (unsigned)((Cout / 64) * (Cin / 64));
        if (Cout % 64 || Cin % 64) pk.tiled = 0;
        *wp = a;
        return TSM_OK;
    };

    // ---- stem
    const int H1 = S / 2, Hp = S / 4, Hs = H1 + 3;
    bf16_t* wp0 = bf ? A.take_n<bf16_t>(64 * 256) : nullptr;
    void* x0 = bf ? A.take((size_t)F * Hs * Hs * 16 * es) : A.take((size_t)F * S * S * 3 * es);
    void* y0 = A.take((size_t)F * H1 * H1 * 64 * es);
    uint8_t* arg0 = A.take_n<uint8_t>((size_t)F * Hp * Hp * 64);
    void* p0 = A.take((size_t)F * Hp * Hp * 64 * es);
    ConvP stem{};
    stem.F = F; stem.T = T; stem.Ho = H1; stem.Wo = H1; stem.Cout = 64; stem.KT = 1; stem.fold = 0;
    if (bf) {
        stem.H = Hs; stem.W = Hs; stem.Cin = 64; stem.pitch = 16; stem.KH = 4; stem.KW = 1; stem.stride = 1; stem.pad = 0;
    } else {
        stem.H = S; stem.W = S; stem.Cin = 3; stem.KH = 7; stem.KW = 7; stem.stride = 2; stem.pad = 3;
    }
    const float *sc0, *sh0;
    bn_slot(&sc0, &sh0);

    // ---- blocks: geometry, weights, BatchNorm slots; activations ping-pong between two buffers
    struct IBlk {
        BlockPlan plan;
        const bf16_t* wp[4];
        const float *sc[4], *sh[4];
    };
    std::vector<IBlk> blks;
    size_t wide_max = (size_t)F * Hp * Hp * 64 * es, mid_max = 0;
    {
        int cin = 64, h = Hp;
        for (const StageSpec& st : kStages) {
            for (int b = 0; b < st.blocks; ++b) {
                const std::string pre = std::string(st.name) + "." + std::to_string(b) + ".";
                tsm_block_desc bd{};
                bd.kind = TSM_BLOCK_BOTTLENECK; bd.N = d->N; bd.T = T; bd.Cin = cin; bd.H = h; bd.W = h;
                bd.Cmid = st.mid; bd.Cout = 4 * st.mid; bd.stride = b == 0 ? st.stride : 1; bd.has_projection = b == 0;
                bd.fold_div = d->fold_div; bd.dtype = dtype; bd.layout = TSM_NTHWC; bd.bn_eps = d->bn_eps;
                IBlk blk;
                TSM_TRY(make_block_plan(&bd, &blk.plan, who));
                const char* cn[3] = {"c1.w", "c2.w", "c3.w"};
                for (int i = 0; i < 3; ++i) {
                    StageDef& sd = blk.plan.st[i];
                    TSM_TRY(pack_conv(pre + cn[i], sd.p.Cout, sd.p.Cin, sd.p.KH, &blk.wp[i]));
                    sd.w = P(pre + cn[i]);
                    bn_slot(&blk.sc[i], &blk.sh[i]);
                    const size_t by = (size_t)sd.p.rows_out() * sd.p.Cout * es;
                    if (i < 2 && by > mid_max) mid_max = by;
                    if (i == 2 && by > wide_max) wide_max = by;
                }
                blk.wp[3] = nullptr; blk.sc[3] = blk.sh[3] = nullptr;
                if (blk.plan.proj) {
                    StageDef& sd = blk.plan.ds;
                    TSM_TRY(pack_conv(pre + "ds.w", sd.p.Cout, sd.p.Cin, 1, &blk.wp[3]));
                    sd.w = P(pre + "ds.w");
                    bn_slot(&blk.sc[3], &blk.sh[3]);
                }
                blks.push_back(blk);
                cin = 4 * st.mid;
                h = blk.plan.st[2].p.Ho;
            }
        }
    }
    void* act[2] = {A.take(wide_max), A.take(wide_max)};
    void* mid[2] = {A.take(mid_max), A.take(mid_max)};
    void* ytmp = A.take(wide_max);    // raw convolution output where the epilogue cannot be fused
    void* scbuf = A.take(wide_max);   // projection shortcut
    const ConvP& lastp = blks.back().plan.st[2].p;
    const int Cf = lastp.Cout, rows_clip = T * lastp.Ho * lastp.Wo;
    float* pm = A.take_n<float>((size_t)d->N * Cf);
    char* scratch_base = dry ? nullptr : (char*)wsp + A.used;
    const size_t scratch_cap = dry ? (size_t)-1 : (ws_bytes > A.used ? ws_bytes - A.used : 0);
    size_t scratch_need = 0;

    // ================= forward =================
    if (!dry) {
        bn_eval_params_kernel<<<dim3(cdiv(nch, 256)), dim3(256), 0, s>>>(bt, params, bn_state, d->bn_eps, scale_all, shift_all);
        LAUNCH_CHECK("bn_eval_params");
        if (bf) {
            if (pk.tiled)
                pack_tiles_kernel<<<dim3(pk.tstart[pk.n]), dim3(256), 0, s>>>(pk, pk, params, pack_base, 0);
            else
                pack_all_kernel<<<dim3(cdiv(pk.start[pk.n], 256)), dim3(256), 0, s>>>(pk, params, pack_base, 0);
            LAUNCH_CHECK("pack_weights_fwd");
            const long total = (long)F * Hs * Hs;
            clips_to_s2d_kernel<<<dim3(cdiv(total, 256)), dim3(256), 0, s>>>((const bf16_t*)clips, (uint4*)x0, S, Hs, total);
            LAUNCH_CHECK("clips_to_s2d");
            stem_pack_kernel<<<dim3(64), dim3(256), 0, s>>>(P("conv1.w"), wp0);
            LAUNCH_CHECK("stem_pack");
        }
    }
    if (bf) {
        RUN(conv_mfma_fwd(stem, (const bf16_t*)x0, wp0, (bf16_t*)y0, nullptr, nullptr, s));
    } else {
        RUN(transpose_frames(clips, x0, F, 3, S * S, 4, s));
        RUN(conv_direct_fwd(stem, dtype, x0, P("conv1.w"), y0, s));
    }
    {
        const int cv = 64 / VEC;
        const long ptotal = (long)F * Hp * Hp * cv;
        if (!dry) {
            if (bf)
                stem_pool_fwd_kernel<bf16_t><<<dim3(cdiv(ptotal, 256)), dim3(256), 0, s>>>((const bf16_t*)y0, sc0, sh0, (bf16_t*)p0, arg0, H1, H1, Hp, Hp, cv, ptotal);
            else
                stem_pool_fwd_kernel<float><<<dim3(cdiv(ptotal, 256)), dim3(256), 0, s>>>((const float*)y0, sc0, sh0, (float*)p0, arg0, H1, H1, Hp, Hp, cv, ptotal);
            LAUNCH_CHECK("stem_pool_fwd");
        }
    }
    const void* cur = p0;
    int flip = 0;
    for (IBlk& b : blks) {
        Arena ws(scratch_base, scratch_cap);
        InferParams ip{};
        for (int i = 0; i < 4; ++i) {
            ip.wp[i] = b.wp[i];
            ip.sc[i] = b.sc[i];
            ip.sh[i] = b.sh[i];
        }
        void* out = act[flip];
        TSM_TRY(block_infer_impl(b.plan, ip, cur, out, mid[0], mid[1], ytmp, scbuf, ws, dry, s));
        if (ws.used > scratch_need) scratch_need = ws.used;
        cur = out;
        flip ^= 1;
    }
    if (!dry) {
        if (bf)
            pool_mean_kernel<bf16_t><<<dim3(cdiv(Cf, 256), d->N), dim3(256), 0, s>>>((const bf16_t*)cur, pm, rows_clip, Cf);
        else
            pool_mean_kernel<float><<<dim3(cdiv(Cf, 128), d->N), dim3(256), 0, s>>>((const float*)cur, pm, rows_clip, Cf);
        LAUNCH_CHECK("pool_mean");
        fc_fwd_kernel<<<dim3(K), dim3(256), 0, s>>>(pm, P("fc.w"), P("fc.b"), logits_out, d->N, Cf, K);
        LAUNCH_CHECK("fc_fwd");
    }
    if (need) *need = align_up(A.used) + align_up(scratch_need) + 256;
    return TSM_OK;
}

extern "C" {

int64_t tsm_resnet50_param_count(int num_classes) {
    if (num_classes <= 0) return 0;
    std::vector<TensorInfo> t = build_table(num_classes);
    return t.back().offset + t.back().count();
}

int tsm_resnet50_num_tensors(void) { return (int)build_table(1).size(); }

int tsm_resnet50_param_info(int num_classes, int index, char* name, int name_cap, int64_t* offset, int* ndim,
                            int shape[4], int* decays) {
    if (num_classes <= 0) return fail(TSM_ERR_SHAPE, "tsm_resnet50_param_info: num_classes must be positive");
    std::vector<TensorInfo> t = build_table(num_classes);
    if (index < 0 || index >= (int)t.size()) return fail(TSM_ERR_SHAPE, "tsm_resnet50_param_info: index %d out of range", index);
    const TensorInfo& ti = t[index];
    if (name && name_cap > 0) {
        strncpy(name, ti.name.c_str(), (size_t)name_cap - 1);
        name[name_cap - 1] = 0;
    }
    if (offset) *offset = ti.offset;
    if (ndim) *ndim = ti.ndim;
    if (shape) for (int i = 0; i < 4; ++i) shape[i] = ti.shape[i];
    if (decays) *decays = ti.decays ? 1 : 0;
    return TSM_OK;
}

int64_t tsm_resnet50_bn_state_count(void) {
    int64_t n = 0;
    for (const TensorInfo& ti : build_table(1))
        if (ti.ndim == 1 && ti.name.size() > 2 && ti.name.compare(ti.name.size() - 2, 2, ".g") == 0) n += 2 * ti.shape[0];
    return n;
}

size_t tsm_resnet50_workspace_bytes(const tsm_r50_desc* d) {
    size_t need = 0;
    if (r50_step(d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, 0, true, nullptr,
                 &need) != TSM_OK)
        return 0;
    return need;
}

int tsm_resnet50_workspace_tensor(const tsm_r50_desc* d, const char* name, size_t* offset, int shape[4], int* elem_bytes) {
    if (!name || !offset || !shape || !elem_bytes) return fail(TSM_ERR_NULLPTR, "tsm_resnet50_workspace_tensor: null pointer");
    WsQuery q{};
    q.name = name;
    TSM_TRY(r50_step(d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, 0, true, nullptr,
                     nullptr, nullptr, &q));
    if (!q.found) return fail(TSM_ERR_UNSUPPORTED, "tsm_resnet50_workspace_tensor: no tensor named '%s'", name);
    *offset = q.offset;
    for (int i = 0; i < 4; ++i) shape[i] = q.shape[i];
    *elem_bytes = q.elem_bytes;
    return TSM_OK;
}

int tsm_resnet50_step(const tsm_r50_desc* d, const void* clips, const int32_t* labels, float* params, float* momentum,
                      float* bn_state, float* grads_out, float* loss_out, float* logits_out, int update, void* ws,
                      size_t ws_bytes, void* stream) {
    return r50_step(d, clips, labels, params, momentum, bn_state, grads_out, loss_out, logits_out, update, ws, ws_bytes,
                    false, (hipStream_t)stream, nullptr);
}

int tsm_resnet50_accum_step(const tsm_r50_desc* d, const void* clips, const int32_t* labels, float* params,
                            float* momentum, float* bn_state, float* grads_accum, float* loss_out, float* logits_out,
                            int micro_index, int micro_count, void* ws, size_t ws_bytes, void* stream) {
    if (micro_count <= 0 || micro_index < 0 || micro_index >= micro_count)
        return fail(TSM_ERR_SHAPE, "tsm_resnet50_accum_step: micro_index %d outside [0, %d)", micro_index, micro_count);
    if (!grads_accum) return fail(TSM_ERR_NULLPTR, "tsm_resnet50_accum_step: null accumulation buffer");
    if (!aligned16(grads_accum)) return fail(TSM_ERR_ALIGN, "tsm_resnet50_accum_step: accumulation buffer must be 16-byte aligned");
    const GradAccum acc = {grads_accum, micro_index, micro_count};
    return r50_step(d, clips, labels, params, momentum, bn_state, nullptr, loss_out, logits_out,
                    micro_index == micro_count - 1, ws, ws_bytes, false, (hipStream_t)stream, nullptr, &acc);
}

// Host-side helper, no GPU work: learning rate of the training recipe at a (fractional) epoch.
double tsm_lr_schedule(double epoch, int total_batch, int warm_batch, double warmup_epochs, double total_epochs) {
    if (total_batch <= 0 || warm_batch <= 0 || !(warmup_epochs >= 0.0) || !(total_epochs > warmup_epochs) || !(epoch >= 0.0)) {
        fail(TSM_ERR_SHAPE, "tsm_lr_schedule: invalid arguments");
        return -1.0;
    }
    const double per_sample = 0.00125 / 8.0;                 // 0.00125 for every 8 samples, scaled linearly
    const double peak = per_sample * total_batch;
    const double start = per_sample * (warm_batch < total_batch ? warm_batch : total_batch);
    if (epoch < warmup_epochs) return start + (peak - start) * (epoch / warmup_epochs);
    if (epoch >= total_epochs) return 0.0;
    const double phase = (epoch - warmup_epochs) / (total_epochs - warmup_epochs);
    return 0.5 * peak * (1.0 + cos(3.14159265358979323846 * phase));
}

size_t tsm_resnet50_infer_workspace_bytes(const tsm_r50_desc* d) {
    size_t need = 0;
    if (r50_infer(d, nullptr, nullptr, nullptr, nullptr, nullptr, 0, true, nullptr, &need) != TSM_OK) return 0;
    return need;
}

int tsm_resnet50_infer(const tsm_r50_desc* d, const void* clips, const float* params, const float* bn_state,
                       float* logits_out, void* ws, size_t ws_bytes, void* stream) {
    return r50_infer(d, clips, params, bn_state, logits_out, ws, ws_bytes, false, (hipStream_t)stream, nullptr);
}

}  // extern "C"
