// bf16 MFMA implicit-GEMM convolutions for gfx950, channels-innermost frames.
//
// The temporal shift of the paper (section 2, Fig. 1) costs nothing here: in
// the forward and weight-gradient kernels it is a per-channel-group offset added
// to the frame index of the input gather (with a zero predicate at the clip
// ends); in the data-gradient kernel its adjoint is a per-channel-group offset
// on the frame index of the output store.  S(x) is never materialised.
//
//   fwd/dgrad  D[M x N] = A[M x K] * B[N x K]^T
//              rows  M = output pixels (all frames), gathered per tap from `src`
//              cols  N = output channels, B = packed weights, K contiguous
//              K     = taps * source channels
//   wgrad      D[Cout x Cin] (per tap) = sum over pixels of dy^T * gathered x
//
// 256 threads = 4 wavefronts of 64; v_mfma_f32_32x32x16_bf16; operands staged
// through LDS with 16-byte loads; fp32 accumulation.
#include "internal.h"

namespace tsm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int BK = 64;        // K elements per main-loop step
static constexpr int LDK = BK + 8;   // LDS row pitch in elements (144 bytes)

struct IgemmArgs {
    const bf16_t* src;     // x (fwd) or dy (dgrad)
    const bf16_t* wp;      // packed weights [N][K]
    bf16_t* dst;           // y (fwd) or dx (dgrad)
    const bf16_t* addend;  // dgrad only: added to dx (nullable)
    float* stats;          // fwd only: per-block partial sums, [gridDim.x][2*Cd] (nullable)
    int F, T;
    int Hs, Ws, Cs;        // source frame
    int Hd, Wd, Cd;        // destination frame; Cd = GEMM N
    int KT, KH, KW;
    int stride;
    int padh, padw;        // fwd: pad; dgrad: K-1-pad
    int fold;              // fwd: shift of source channels; dgrad: adjoint shift of destination channels
    long M;
    int K;
    int mtiles, ntiles;
};

__device__ __forceinline__ int group_dt(int c, int fold) { return c < fold ? 1 : (c < 2 * fold ? -1 : 0); }

template <int BM, int BN, int WM, int WN, bool DGRAD>
__global__ void __launch_bounds__(256, 2) igemm_kernel(IgemmArgs a) {
    static_assert(WM * WN == 4, "four wavefronts");
    constexpr int TM = BM / WM, TN = BN / WN;       // wavefront tile
    constexpr int MI = TM / 32, NJ = TN / 32;       // 32x32 MFMA tiles per wavefront
    constexpr int KV = BK / 8;                      // 16-byte vectors per tile row
    constexpr int RPP = 256 / KV;                   // tile rows loaded per pass
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int LDC = BN + 8;                     // staging pitch (elements)
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile / thread mismatch");
    static_assert(BM * LDC <= 2 * (BM + BN) * LDK, "staging must fit in the operand buffers");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* As = (bf16_t*)smem;                      // [2][BM][LDK]
    bf16_t* Bs = As + 2 * BM * LDK;                  // [2][BN][LDK]
    bf16_t* Cst = (bf16_t*)smem;                     // [BM][LDC], reuses As/Bs after the main loop
    float* s_sum = (float*)(Bs + 2 * BN * LDK);      // [Cd] then [Cd]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int kvec = tid % KV, lrow = tid / KV;
    const bool do_stats = (!DGRAD) && a.stats != nullptr;

    if (do_stats) {
        for (int c = tid; c < 2 * a.Cd; c += 256) s_sum[c] = 0.f;
    }
    __syncthreads();

    const int hw_d = a.Hd * a.Wd;
    const int nk = (a.K + BK - 1) / BK;
    const int total_tiles = ((a.mtiles + 7) / 8) * 8 * a.ntiles;  // M tiles padded to whole groups of 8

    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        // Tiles that share an M range sit on the same XCD (ids 8 apart) so the
        // gathered rows are served by that XCD's L2.
        const int xcd = tile & 7, slot = tile >> 3;
        int mt = (slot / a.ntiles) * 8 + xcd;
        int nt = slot % a.ntiles;
        if (mt >= a.mtiles) continue;  // the last group of 8 M tiles may be ragged (block-uniform branch)
        const long m0 = (long)mt * BM;
        const int n0 = nt * BN;

        // ---- decode this thread's A rows once per tile
        int rf[PA], rt[PA], rh[PA], rw[PA];
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const long m = m0 + i * RPP + lrow;
            if (m < a.M) {
                const int f = (int)(m / hw_d);
                const int pix = (int)(m - (long)f * hw_d);
                const int dh = pix / a.Wd, dw = pix - dh * a.Wd;
                rf[i] = f;
                rt[i] = f % a.T;
                rh[i] = (DGRAD ? dh : dh * a.stride) - a.padh;
                rw[i] = (DGRAD ? dw : dw * a.stride) - a.padw;
            } else {
                rf[i] = -1;
                rt[i] = rh[i] = rw[i] = 0;
            }
        }

        f32x16 acc[MI][NJ];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        u32x4 areg[PA], breg[PB];

        auto load_tiles = [&](int kc) {
            const int kk = kc * BK + kvec * 8;
            const bool kvalid = kk < a.K;
            const int tap = kk / a.Cs;
            const int c = kk - tap * a.Cs;
            const int kw = tap % a.KW;
            const int kh = (tap / a.KW) % a.KH;
            const int kt = tap / (a.KW * a.KH);
            const int df = kt - a.KT / 2 + (DGRAD ? 0 : group_dt(c, a.fold));
#pragma unroll
            for (int i = 0; i < PA; ++i) {
                int sh = rh[i] + kh, sw = rw[i] + kw;
                bool ok = kvalid && rf[i] >= 0;
                if (DGRAD && a.stride > 1) {
                    ok = ok && sh >= 0 && sw >= 0 && (sh % a.stride == 0) && (sw % a.stride == 0);
                    sh /= a.stride;
                    sw /= a.stride;
                }
                const int ts = rt[i] + df;
                ok = ok && ts >= 0 && ts < a.T && sh >= 0 && sh < a.Hs && sw >= 0 && sw < a.Ws;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (ok) {
                    const long off = (((long)(rf[i] + df) * a.Hs + sh) * a.Ws + sw) * a.Cs + c;
                    v = *(const u32x4*)(a.src + off);
                }
                areg[i] = v;
            }
#pragma unroll
            for (int j = 0; j < PB; ++j) {
                const int n = n0 + j * RPP + lrow;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (kvalid && n < a.Cd) v = *(const u32x4*)(a.wp + (long)n * a.K + kk);
                breg[j] = v;
            }
        };
        auto store_tiles = [&](int buf) {
            bf16_t* Ab = As + buf * BM * LDK;
            bf16_t* Bb = Bs + buf * BN * LDK;
#pragma unroll
            for (int i = 0; i < PA; ++i) *(u32x4*)(Ab + (i * RPP + lrow) * LDK + kvec * 8) = areg[i];
#pragma unroll
            for (int j = 0; j < PB; ++j) *(u32x4*)(Bb + (j * RPP + lrow) * LDK + kvec * 8) = breg[j];
        };

        load_tiles(0);
        store_tiles(0);
        __syncthreads();
        for (int kc = 0; kc < nk; ++kc) {
            const int buf = kc & 1;
            if (kc + 1 < nk) load_tiles(kc + 1);
            const bf16_t* Ab = As + buf * BM * LDK + (wm * TM + (lane & 31)) * LDK + 8 * (lane >> 5);
            const bf16_t* Bb = Bs + buf * BN * LDK + (wn * TN + (lane & 31)) * LDK + 8 * (lane >> 5);
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8 af[MI], bfr[NJ];
#pragma unroll
                for (int i = 0; i < MI; ++i) af[i] = *(const bf16x8*)(Ab + i * 32 * LDK + ks * 16);
#pragma unroll
                for (int j = 0; j < NJ; ++j) bfr[j] = *(const bf16x8*)(Bb + j * 32 * LDK + ks * 16);
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            }
            if (kc + 1 < nk) store_tiles(buf ^ 1);
            __syncthreads();
        }

        // ---- epilogue: round to bf16, per-channel statistics, stage through LDS, 16-byte stores.
        // D layout of the 32x32 MFMA: lane holds column (lane % 32); register r holds
        // row 8*(r/4) + 4*(lane/32) + r%4.
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float s1 = 0.f, s2 = 0.f;
            const int col = wn * TN + j * 32 + (lane & 31);
#pragma unroll
            for (int i = 0; i < MI; ++i) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const bf16_t b = f32_to_bf16(acc[i][j][r]);
                    const int row = wm * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    Cst[row * LDC + col] = b;
                    if (do_stats) {
                        const float v = bf16_to_f32(b);
                        s1 += v;
                        s2 = fmaf(v, v, s2);
                    }
                }
            }
            if (do_stats && n0 + col < a.Cd) {
                atomicAdd(&s_sum[n0 + col], s1);
                atomicAdd(&s_sum[a.Cd + n0 + col], s2);
            }
        }
        __syncthreads();
        {
            constexpr int CV = BN / 8;          // vectors per staged row
            constexpr int RPS = 256 / CV;       // rows per pass
            const int vcol = tid % CV, r0 = tid / CV;
            const int col = n0 + vcol * 8;
#pragma unroll
            for (int pss = 0; pss < BM / RPS; ++pss) {
                const int row = pss * RPS + r0;
                const long m = m0 + row;
                if (m >= a.M || col >= a.Cd) continue;
                u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
                if (!DGRAD) {
                    *(u32x4*)(a.dst + m * a.Cd + col) = v;
                } else {
                    const int dt = group_dt(col, a.fold);
                    const int t = (int)((m / hw_d) % a.T);
                    auto emit = [&](long mrow, bool with_value) {
                        u32x4 o = with_value ? v : u32x4{0u, 0u, 0u, 0u};
                        if (a.addend) {
                            const u32x4 ad = *(const u32x4*)(a.addend + mrow * a.Cd + col);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const float lo = bf16_to_f32((bf16_t)(o[q] & 0xffffu)) + bf16_to_f32((bf16_t)(ad[q] & 0xffffu));
                                const float hi = bf16_to_f32((bf16_t)(o[q] >> 16)) + bf16_to_f32((bf16_t)(ad[q] >> 16));
                                o[q] = (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
                            }
                        }
                        *(u32x4*)(a.dst + mrow * a.Cd + col) = o;
                    };
                    if (dt == 0) {
                        emit(m, true);
                    } else {
                        if (t + dt >= 0 && t + dt < a.T) emit(m + (long)dt * hw_d, true);
                        // the frame that receives nothing from inside the clip
                        if ((dt == 1 && t == 0) || (dt == -1 && t == a.T - 1)) emit(m, false);
                    }
                }
            }
        }
        __syncthreads();
    }

    if (do_stats) {   // every block publishes its row, zeros included: the consumer adds all rows up
        __syncthreads();
        float* prow = a.stats + (size_t)blockIdx.x * 2 * a.Cd;
        for (int c = tid; c < 2 * a.Cd; c += 256) prow[c] = s_sum[c];
    }
}

// ---------------------------------------------------------------------------------
static int g_num_cu = 0;
static int num_cu() {
    if (g_num_cu == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            g_num_cu = prop.multiProcessorCount;
        if (g_num_cu <= 0) g_num_cu = 256;
    }
    return g_num_cu;
}

bool mfma_conv_supported(const ConvP& p) {
    if (p.Cin % 8 || p.Cout % 8) return false;
    if (p.fold % 8) return false;
    if (p.Cin > 8192 || p.Cout > 8192) return false;
    if (p.K() > 0x3fffffffL || p.rows_in() * p.Cin > 0x7fffffffffffL) return false;
    return true;
}

// Persistent grid: two blocks per CU (a multiple of 8 so that a block stays on one XCD), capped by
// the number of tile ids, which enumerate (group of 8 M tiles) x N tiles x (xcd).
static int igemm_grid(long M, int Cd, int BM, int BN) {
    const int mtiles = (int)((M + BM - 1) / BM), ntiles = (Cd + BN - 1) / BN;
    const int total = ((mtiles + 7) / 8) * 8 * ntiles;
    int grid = 2 * num_cu();
    grid = (grid / 8) * 8;
    if (grid > total) grid = total;
    if (grid < 1) grid = 1;
    return grid;
}

template <int BM, int BN, int WM, int WN, bool DGRAD>
static int launch_igemm(IgemmArgs& a, hipStream_t s) {
    a.mtiles = (int)((a.M + BM - 1) / BM);
    a.ntiles = (a.Cd + BN - 1) / BN;
    size_t smem = (size_t)2 * (BM + BN) * LDK * sizeof(bf16_t) + (size_t)2 * a.Cd * sizeof(float);
    auto kern = igemm_kernel<BM, BN, WM, WN, DGRAD>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "igemm: cannot raise dynamic LDS limit");
        configured = true;
    }
    const int grid = igemm_grid(a.M, a.Cd, BM, BN);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, s, a);
    // class names carry the tile shape so that they map one-to-one onto kernel symbols
    return check_launch(DGRAD ? (BN == 64 ? "igemm_dgrad_128x64" : "igemm_dgrad_128x128")
                              : (BN == 64 ? "igemm_fwd_128x64" : "igemm_fwd_128x128"));
}

template <bool DGRAD>
static int dispatch_igemm(IgemmArgs& a, hipStream_t s) {
    if (a.M == 0) return TSM_OK;
    if (a.Cd <= 64) return launch_igemm<128, 64, 4, 1, DGRAD>(a, s);
    return launch_igemm<128, 128, 2, 2, DGRAD>(a, s);
}

int conv_mfma_fwd_blocks(const ConvP& p) { return igemm_grid(p.rows_out(), p.Cout, 128, p.Cout <= 64 ? 64 : 128); }

int conv_mfma_fwd(const ConvP& p, const bf16_t* x, const bf16_t* wp, bf16_t* y, float* stats, hipStream_t s) {
    IgemmArgs a;
    a.src = x; a.wp = wp; a.dst = y; a.addend = nullptr; a.stats = stats;
    a.F = p.F; a.T = p.T;
    a.Hs = p.H; a.Ws = p.W; a.Cs = p.Cin;
    a.Hd = p.Ho; a.Wd = p.Wo; a.Cd = p.Cout;
    a.KT = p.KT; a.KH = p.KH; a.KW = p.KW;
    a.stride = p.stride; a.padh = p.pad; a.padw = p.pad;
    a.fold = p.fold;
    a.M = p.rows_out();
    a.K = (int)p.K();
    return dispatch_igemm<false>(a, s);
}

int conv_mfma_dgrad(const ConvP& p, const bf16_t* dy, const bf16_t* wd, bf16_t* dx, const bf16_t* addend,
                    hipStream_t s) {
    IgemmArgs a;
    a.src = dy; a.wp = wd; a.dst = dx; a.addend = addend; a.stats = nullptr;
    a.F = p.F; a.T = p.T;
    a.Hs = p.Ho; a.Ws = p.Wo; a.Cs = p.Cout;
    a.Hd = p.H; a.Wd = p.W; a.Cd = p.Cin;
    a.KT = p.KT; a.KH = p.KH; a.KW = p.KW;
    a.stride = p.stride; a.padh = p.KH - 1 - p.pad; a.padw = p.KW - 1 - p.pad;
    a.fold = p.fold;
    a.M = p.rows_in();
    a.K = p.taps() * p.Cout;
    return dispatch_igemm<true>(a, s);
}

// ---------------------------------------------------------------------------------
// Weight gradient, D[Cout x K] = dy^T [Cout x pixels] * gathered x [pixels x K] with
// K = taps * Cin enumerated tap-major (the packed-weight order).  Per block: a
// [BCO x BCI] tile of D reduced over a chunk of output pixels, added with fp32
// atomics to dw in the ABI order [Cout][Cin][taps].  Both operands are needed with the pixel index contiguous, so the
// 16-byte global rows ([pixel][channel]) are transposed on their way into LDS:
// each thread pairs two consecutive pixels of eight channels into eight 32-bit
// LDS writes.
struct WgradArgs {
    const bf16_t* x;
    const bf16_t* dy;
    float* dw;             // element (co, ci, tap) at co*so + ci*si + tap*st
    long so;
    int si, st, cin_real;
    int F, T;
    int H, W, Cin;
    int Ho, Wo, Cout;
    int KT, KH, KW, stride, pad;
    int fold;
    long M;                // output pixels
    long chunk;            // pixels per block (multiple of 64)
    int K;                 // taps * Cin
    int col_tiles;
};

static constexpr int WMK = 64;        // pixels per main-loop step
static constexpr int LDT = WMK + 8;   // pitch of the transposed tiles

// Element offset of pixel pair `pp` (two pixels = one 32-bit word) in the transposed
// tile row `row`: groups of four words (one 16-byte fragment) are XOR-swizzled with
// the row's channel-vector index so that the eight lanes writing eight channel vectors
// of the same pixels fall into different LDS banks.
__device__ __forceinline__ int swz_pair(int pp, int row) { return ((((pp >> 2) ^ ((row >> 3) & 7)) << 2) | (pp & 3)) * 2; }
// Element offset of the 8-pixel fragment `g` (0..7) of row `row`.
__device__ __forceinline__ int swz_frag(int g, int row) { return (g ^ ((row >> 3) & 7)) * 8; }

template <int BCO, int BCI>
__global__ void __launch_bounds__(256, 2) wgrad_kernel(WgradArgs a) {
    constexpr int TM = BCO / 2, TN = BCI / 2;
    constexpr int MI = TM / 32, NJ = TN / 32;
    __shared__ __attribute__((aligned(16))) bf16_t At[2][BCO][LDT];   // dy^T  [co][pixel]
    __shared__ __attribute__((aligned(16))) bf16_t Bt[2][BCI][LDT];   // xs^T  [column][pixel]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int co0 = (blockIdx.y / a.col_tiles) * BCO;
    const int j0 = (blockIdx.y % a.col_tiles) * BCI;
    const long mbeg = (long)blockIdx.x * a.chunk;
    long mend = mbeg + a.chunk;
    if (mend > a.M) mend = a.M;
    const int hw = a.Ho * a.Wo;

    // loader mapping: consecutive lanes read consecutive 16-byte pieces of one row;
    // every thread owns pixel pairs (2*pp, 2*pp+1) of channel vector `vec`.
    constexpr int AV = BCO / 8, BV = BCI / 8;         // vectors per row
    constexpr int AP = (32 * AV + 255) / 256;         // (pair, vec) items per thread
    constexpr int BP = (32 * BV + 255) / 256;

    // this thread's B columns: 8 consecutive K indices = 8 channels of one tap
    int b_ci[BP], b_kh[BP], b_kw[BP], b_df[BP];
#pragma unroll
    for (int q = 0; q < BP; ++q) {
        const int vec = (q * 256 + tid) % BV;
        const int j = j0 + vec * 8;
        if (j < a.K) {
            const int tap = j / a.Cin;
            b_ci[q] = j - tap * a.Cin;
            b_kw[q] = tap % a.KW;
            b_kh[q] = (tap / a.KW) % a.KH;
            b_df[q] = tap / (a.KW * a.KH) - a.KT / 2 + group_dt(b_ci[q], a.fold);
        } else {
            b_ci[q] = -1;
            b_kh[q] = b_kw[q] = b_df[q] = 0;
        }
    }

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 ar[AP][2], br[BP][2];

    auto load = [&](long mstep) {
#pragma unroll
        for (int q = 0; q < AP; ++q) {
            const int item = q * 256 + tid;
            const int vec = item % AV, pp = item / AV;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const long m = mstep + 2 * pp + h;
                const int co = co0 + vec * 8;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (pp < 32 && m < mend && co < a.Cout) v = *(const u32x4*)(a.dy + m * a.Cout + co);
                ar[q][h] = v;
            }
        }
#pragma unroll
        for (int q = 0; q < BP; ++q) {
            const int pp = (q * 256 + tid) / BV;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const long m = mstep + 2 * pp + h;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (pp < 32 && m < mend && b_ci[q] >= 0) {
                    const int f = (int)(m / hw);
                    const int pix = (int)(m - (long)f * hw);
                    const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
                    const int ih = oh * a.stride + b_kh[q] - a.pad, iw = ow * a.stride + b_kw[q] - a.pad;
                    const int ts = f % a.T + b_df[q];
                    if (ts >= 0 && ts < a.T && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W)
                        v = *(const u32x4*)(a.x + (((long)(f + b_df[q]) * a.H + ih) * a.W + iw) * a.Cin + b_ci[q]);
                }
                br[q][h] = v;
            }
        }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int q = 0; q < AP; ++q) {
            const int item = q * 256 + tid;
            const int vec = item % AV, pp = item / AV;
            if (pp < 32) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t lo = ar[q][0][e], hi = ar[q][1][e];
                    *(uint32_t*)&At[buf][vec * 8 + 2 * e][swz_pair(pp, vec * 8)] = (lo & 0xffffu) | (hi << 16);
                    *(uint32_t*)&At[buf][vec * 8 + 2 * e + 1][swz_pair(pp, vec * 8)] = (lo >> 16) | (hi & 0xffff0000u);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < BP; ++q) {
            const int item = q * 256 + tid;
            const int vec = item % BV, pp = item / BV;
            if (pp < 32) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t lo = br[q][0][e], hi = br[q][1][e];
                    *(uint32_t*)&Bt[buf][vec * 8 + 2 * e][swz_pair(pp, vec * 8)] = (lo & 0xffffu) | (hi << 16);
                    *(uint32_t*)&Bt[buf][vec * 8 + 2 * e + 1][swz_pair(pp, vec * 8)] = (lo >> 16) | (hi & 0xffff0000u);
                }
            }
        }
    };

    if (mbeg < mend) {
        const int nsteps = (int)((mend - mbeg + WMK - 1) / WMK);
        load(mbeg);
        store(0);
        __syncthreads();
        for (int st = 0; st < nsteps; ++st) {
            const int buf = st & 1;
            if (st + 1 < nsteps) load(mbeg + (long)(st + 1) * WMK);
#pragma unroll
            for (int ks = 0; ks < WMK / 16; ++ks) {
                bf16x8 af[MI], bfr[NJ];
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int row = wm * TM + i * 32 + (lane & 31);
                    af[i] = *(const bf16x8*)&At[buf][row][swz_frag(2 * ks + (lane >> 5), row)];
                }
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int row = wn * TN + j * 32 + (lane & 31);
                    bfr[j] = *(const bf16x8*)&Bt[buf][row][swz_frag(2 * ks + (lane >> 5), row)];
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            }
            if (st + 1 < nsteps) store(buf ^ 1);
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int col = j0 + wn * TN + j * 32 + (lane & 31);
                const int tap = col / a.Cin, ci = col - tap * a.Cin;
                if (col >= a.K || ci >= a.cin_real) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int co = co0 + wm * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (co < a.Cout) atomicAdd(a.dw + (long)co * a.so + (long)ci * a.si + (long)tap * a.st, acc[i][j][r]);
                }
            }
    }
}

int conv_mfma_wgrad(const ConvP& p, const bf16_t* x, const bf16_t* dy, float* dw, int cin_real, bool packed,
                    hipStream_t s) {
    WgradArgs a;
    a.x = x; a.dy = dy; a.dw = dw; a.cin_real = cin_real;
    if (packed) {   // [Cout][taps][p.Cin]: consecutive lanes (channels) hit consecutive addresses
        a.so = (long)p.taps() * p.Cin; a.si = 1; a.st = p.Cin;
    } else {        // ABI order [Cout][cin_real][taps]
        a.so = (long)cin_real * p.taps(); a.si = p.taps(); a.st = 1;
    }
    a.F = p.F; a.T = p.T; a.H = p.H; a.W = p.W; a.Cin = p.Cin;
    a.Ho = p.Ho; a.Wo = p.Wo; a.Cout = p.Cout;
    a.KT = p.KT; a.KH = p.KH; a.KW = p.KW; a.stride = p.stride; a.pad = p.pad;
    a.fold = p.fold;
    a.M = p.rows_out();
    a.K = (int)p.K();
    if (a.M == 0) return TSM_OK;
    const bool big = p.Cout > 64 && a.K > 64;
    const int bco = big ? 128 : 64, bci = big ? 128 : 64;
    a.col_tiles = cdiv(a.K, bci);
    const int tiles = cdiv(p.Cout, bco) * a.col_tiles;
    long want = (long)4 * num_cu() / tiles;
    if (want < 1) want = 1;
    long chunk = (a.M + want - 1) / want;
    chunk = (chunk + WMK - 1) / WMK * WMK;
    if (chunk < 4 * WMK) chunk = 4 * WMK;
    a.chunk = chunk;
    const unsigned gx = (unsigned)((a.M + chunk - 1) / chunk);
    dim3 grid(gx, (unsigned)tiles);
    if (big)
        wgrad_kernel<128, 128><<<grid, dim3(256), 0, s>>>(a);
    else
        wgrad_kernel<64, 64><<<grid, dim3(256), 0, s>>>(a);
    return check_launch(big ? "wgrad_128x128" : "wgrad_64x64");
}

}  // namespace tsm
