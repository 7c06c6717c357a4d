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
// v_mfma_f32_32x32x16_bf16, operands staged through LDS, fp32 accumulation.  Kernels:
//   igemm_ring_kernel  fwd/dgrad, source channels % 64 == 0: 256 x {128,64} tile, eight wavefronts,
//                      buffer-load gathers, loads and LDS stores spread over the MFMA groups
//   conv3x3_c64_kernel fwd/dgrad, 3x3 stride 1, 64 -> 64 channels, many tiles: weights and the tile's input patch
//                      resident in LDS, no barrier inside a tile's main loop
//   stem_s2d_kernel    fwd of the stem in space-to-depth form, many tiles: the same scheme for its 4-row window
//   igemm_kernel       fwd/dgrad, any channel count % 8 == 0: 128 x {128,64} tile, four wavefronts,
//                      register prefetch (the fallback)
//   wgrad_tr_kernel    wgrad, channels % 64 == 0: operands read with the transposing LDS load
//   wgrad_kernel       wgrad, any channel count % 8 == 0: operands transposed in registers (the fallback)
#include <stdlib.h>
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
    // igemm_ring_kernel only: with add_stride == 2 the addend holds only the destination pixels whose row and
    // column are even, densely, as [F][add_ho][add_wo][Cd] (the data gradient of a 1x1 stride-2 projection:
    // everything else is structurally zero and is neither stored nor read)
    int add_stride, add_ho, add_wo;
    float* stats;          // per-block partial sums, [gridDim.x][2*Cd] (nullable): fwd: sum and sum of squares of
                           // y; dgrad with `act`: the two BatchNorm-backward sums of the masked gradient
    // dgrad, igemm_ring_kernel only (nullable): dst is the gradient w.r.t. act = ReLU(BatchNorm(ybn)).  The
    // epilogue then zeroes it where act <= 0 and accumulates, per channel, sum(dz) and sum(dz * (ybn - mean) * rstd).
    const bf16_t* act;
    const bf16_t* ybn;
    const float* bn_mean;
    const float* bn_rstd;
    const uint8_t* act_bits;   // igemm_ring_kernel, MBITS variants: the decisions act > 0 as bits, [rows][Cd/8]
    // fwd, igemm_ring_kernel only (nullable): the stored result is act(ep_scale[c]*y + ep_shift[c] + ep_res), y
    // rounded to bf16 first; ep_res (nullable) has the shape of dst; act = ReLU when ep_relu, identity otherwise.
    // This is BatchNorm with known statistics (inference) folded into the epilogue.
    const float* ep_scale;
    const float* ep_shift;
    const bf16_t* ep_res;
    int ep_relu;
    int F, T;
    int Hs, Ws, Cs;        // source frame
    int pitch;             // elements between consecutive source pixels (Cs, or less: see ConvP::pitch)
    int Hd, Wd, Cd;        // destination frame; Cd = GEMM N
    int KT, KH, KW;
    int stride;
    int padh, padw;        // fwd: pad; dgrad: K-1-pad
    int fold;              // fwd: shift of source channels; dgrad: adjoint shift of destination channels
    int K;                 // taps * Cs: row pitch of wp
    int ntiles;            // tiles along N
    // Destination pixels are processed in classes.  Forward and stride-1 dgrad have one class (all
    // pixels, all taps).  A stride-s dgrad has s*s parity classes: pixel (dh, dw) with dh % s == ph,
    // dw % s == pw receives only the flipped taps a = a0h + th*s, b = a0w + tw*s, so each class is a
    // dense GEMM over its own tap subset and no multiply is spent on structural zeros.
    int ncls, cstep;
    int ph[4], pw[4];      // parity of the class
    int hc[4], wc[4];      // pixels of that parity per frame
    int mt0[5];            // prefix sum of M tiles per class
    int a0h[4], nth[4], a0w[4], ntw[4];
};

__device__ __forceinline__ int group_dt(int c, int fold) { return c < fold ? 1 : (c < 2 * fold ? -1 : 0); }

// quad_perm [1,0,3,2]: every lane reads its neighbour in the pair (lane ^ 1)
__device__ __forceinline__ uint32_t pair_swap(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);
}

// Lanes whose gather falls on padding (spatial border, clip end, K tail, row beyond M) read this instead.
static __device__ uint4 g_zero_page[1];

// Per tile row, decoded once per tile into LDS:
//   off   element offset in `src` of the row's tap origin (frame f, source row oh, column ow); may point
//         before the frame when the origin lies in the padding -- it is only used for taps inside the frame
//   mask  bits 0..7: tap rows th with 0 <= oh+th < Hs; bits 8..15: tap columns tw with 0 <= ow+tw < Ws;
//         bit 30: frame t+1 is in the clip; bit 31: frame t-1 is in the clip; 0 for rows beyond M
//   dst   destination row index, -1 for rows beyond M
struct RowInfo {
    long off;
    uint32_t mask;
    int dst;
};

// PF: K steps of gathered data kept in flight in registers (1 or 2); MINB: blocks per CU the register
// budget is sized for (2: 256 registers per lane, 1: 512).
template <int BM, int BN, int WM, int WN, bool DGRAD, int PF, int MINB>
__global__ void __launch_bounds__(256, MINB) igemm_kernel(IgemmArgs a) {
    static_assert(WM * WN == 4, "four wavefronts");
    constexpr int TM = BM / WM, TN = BN / WN;       // wavefront tile
    constexpr int MI = TM / 32, NJ = TN / 32;       // 32x32 MFMA tiles per wavefront
    constexpr int KV = BK / 8;                      // 16-byte vectors per tile row
    constexpr int RPP = 256 / KV;                   // tile rows loaded per pass
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int LDC = BN + 8;                     // staging pitch (elements)
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile / thread mismatch");
    static_assert(BM * LDC <= 2 * (BM + BN) * LDK, "staging must fit in the operand buffers");
    static_assert(sizeof(RowInfo) == 16, "one 16-byte LDS read per row");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* As = (bf16_t*)smem;                      // [2][BM][LDK]
    bf16_t* Bs = As + 2 * BM * LDK;                  // [2][BN][LDK]
    bf16_t* Cst = (bf16_t*)smem;                     // [BM][LDC], reuses As/Bs after the main loop
    RowInfo* s_row = (RowInfo*)(Bs + 2 * BN * LDK);  // [2][BM]: rows of the current and of the next tile
    // per-tile statistics slots [2 stats][WM*2 slots][BN], placed behind the staging tile in the operand buffers
    float* s_part = (float*)(Cst + BM * LDC);
    static_assert((size_t)BM * LDC * 2 + (size_t)2 * WM * 2 * BN * 4 <= (size_t)2 * (BM + BN) * LDK * 2, "slots must fit");

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int kvec = tid % KV, lrow = tid / KV;
    const bool do_stats = (!DGRAD) && a.stats != nullptr;
    const bool uniform_tap = (a.Cs % BK) == 0;      // a K step never straddles two taps
    const bf16_t* zero_page = (const bf16_t*)g_zero_page;

    // Statistics: this block owns one row of the partial buffer.  It is zeroed here; after every tile one
    // fixed thread per column adds that tile's column sums to it (device-scope atomics used as plain
    // coherent read-modify-writes: no other block touches the row), in tile order -- so the result is
    // bit-reproducible.
    float* prow = do_stats ? a.stats + (size_t)blockIdx.x * 2 * a.Cd : nullptr;
    if (do_stats) {
        // the barrier below waits for these stores to be acknowledged by L2, where the later atomics execute
        for (int c = tid; c < 2 * a.Cd; c += 256) prow[c] = 0.f;
    }

    const int hw_d = a.Hd * a.Wd;
    const int hw_s = a.Hs * a.Ws;
    const int frame_el = hw_s * a.Cs;               // elements per source frame
    const int mtiles = a.mt0[a.ncls];
    const int total_tiles = ((mtiles + 7) / 8) * 8 * a.ntiles;  // M tiles padded to whole groups of 8

    // Tile ids: tiles that share an M range sit on the same XCD (ids 8 apart) so the gathered rows are
    // served by that XCD's L2.  The last group of 8 M tiles may be ragged: such ids are skipped.
    auto tile_mt = [&](int tile) { return ((tile >> 3) / a.ntiles) * 8 + (tile & 7); };
    auto next_tile = [&](int tile) {
        while (tile < total_tiles && tile_mt(tile) >= mtiles) tile += gridDim.x;
        return tile < total_tiles ? tile : -1;
    };

    // Everything the main loop needs to know about one tile.
    struct Ctx {
        int n0, nth, ntw, a0h, a0w, ntaps, nk;
        const bf16_t* aptr[PA];
        uint32_t amask[PA];
        const bf16_t* bptr[PB];
        // position of the next K step to fetch: class-local tap (kt, th, tw), first channel of this
        // thread's 16-byte vector, flat tap index; advanced by load_tiles without any division
        int kt, th, tw, ch, ltap;
    };

    // ---- decode a tile's rows, one row per thread, into LDS row buffer rb
    auto decode_rows = [&](int tile, int rb) {
        if (tid < BM) {
            const int mt = tile_mt(tile);
            int cls = 0;
            while (cls + 1 < a.ncls && mt >= a.mt0[cls + 1]) ++cls;
            const int hc = a.hc[cls], wc = a.wc[cls];
            const long Mc = (long)a.F * hc * wc;
            const long m = (long)(mt - a.mt0[cls]) * BM + tid;
            RowInfo info;
            info.off = 0;
            info.mask = 0;
            info.dst = -1;
            if (m < Mc) {
                const int f = (int)(m / (hc * wc));
                const int q = (int)(m - (long)f * (hc * wc));
                const int qh = q / wc, qw = q - qh * wc;
                const int dh = qh * a.cstep + a.ph[cls], dw = qw * a.cstep + a.pw[cls];
                // source coordinate of class-local tap (th, tw) is (oh + th, ow + tw); for a strided dgrad
                // the division by the stride is exact by construction of the class
                const int oh = DGRAD ? (dh - a.padh + a.a0h[cls]) / a.cstep : dh * a.stride - a.padh;
                const int ow = DGRAD ? (dw - a.padw + a.a0w[cls]) / a.cstep : dw * a.stride - a.padw;
                const int t = f % a.T;
                uint32_t mask = 0;
                for (int th = 0; th < a.nth[cls]; ++th)
                    if (oh + th >= 0 && oh + th < a.Hs) mask |= 1u << th;
                for (int tw = 0; tw < a.ntw[cls]; ++tw)
                    if (ow + tw >= 0 && ow + tw < a.Ws) mask |= 1u << (8 + tw);
                if (t + 1 < a.T) mask |= 1u << 30;
                if (t >= 1) mask |= 1u << 31;
                info.off = ((long)f * hw_s + (long)oh * a.Ws + ow) * a.Cs;
                info.mask = mask;
                info.dst = (f * a.Hd + dh) * a.Wd + dw;
            }
            s_row[rb * BM + tid] = info;
        }
    };
    // ---- per-thread view of a decoded tile (call after the barrier that follows decode_rows)
    auto make_ctx = [&](int tile, int rb) {
        Ctx c;
        const int mt = tile_mt(tile);
        int cls = 0;
        while (cls + 1 < a.ncls && mt >= a.mt0[cls + 1]) ++cls;
        c.n0 = ((tile >> 3) % a.ntiles) * BN;
        c.nth = a.nth[cls]; c.ntw = a.ntw[cls]; c.a0h = a.a0h[cls]; c.a0w = a.a0w[cls];
        c.ntaps = a.KT * c.nth * c.ntw;
        c.nk = (c.ntaps * a.Cs + BK - 1) / BK;
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const RowInfo ri = s_row[rb * BM + i * RPP + lrow];
            c.aptr[i] = a.src + ri.off;
            c.amask[i] = ri.mask;
        }
#pragma unroll
        for (int j = 0; j < PB; ++j) {
            const int n = c.n0 + j * RPP + lrow;
            c.bptr[j] = n < a.Cd ? a.wp + (long)n * a.K : nullptr;
        }
        c.kt = c.th = c.tw = c.ltap = 0;
        c.ch = kvec * 8;
        while (c.ch >= a.Cs) {   // fewer than 64 channels: this thread's vector starts in a later tap
            c.ch -= a.Cs;
            ++c.ltap;
            if (++c.tw >= c.ntw) { c.tw = 0; if (++c.th >= c.nth) { c.th = 0; ++c.kt; } }
        }
        return c;
    };

    // gathered data in flight: one K step, or two (PF2: steps k+1 and k+2) when the registers allow it
    constexpr bool PF2 = (PF == 2);
    u32x4 areg[PA], breg[PB], areg1[PF2 ? PA : 1], breg1[PF2 ? PB : 1];

    // Fetches the next K step of tile `c` (steps are fetched strictly in order) and advances c's position.
    auto load_tiles = [&](Ctx& c, u32x4* areg, u32x4* breg) {
        // steps beyond the tile's K range (harmless filler loads) read the zero page
        const bool kvalid = c.ltap < c.ntaps;
        const int ch = c.ch, th_ = c.th, tw_ = c.tw, kt = c.kt;
        const int d = kt - a.KT / 2 + (DGRAD ? 0 : group_dt(ch, a.fold));   // frame offset, in {-1, 0, 1}
        // bits a row's mask must have for this tap
        const uint32_t need = (1u << th_) | (1u << (8 + tw_)) | (d > 0 ? 1u << 30 : 0u) | (d < 0 ? 1u << 31 : 0u);
        const int aoff = d * frame_el + (th_ * a.Ws + tw_) * a.Cs + ch;
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const bool ok = kvalid && (c.amask[i] & need) == need;
            const bf16_t* p = ok ? c.aptr[i] + aoff : zero_page;
            areg[i] = *(const u32x4*)p;
        }
        const int ta = c.a0h + th_ * a.cstep, tb = c.a0w + tw_ * a.cstep;   // (flipped) tap coordinates
        const int woff = ((kt * a.KH + ta) * a.KW + tb) * a.Cs + ch;
#pragma unroll
        for (int j = 0; j < PB; ++j) {
            const bf16_t* p = (kvalid && c.bptr[j]) ? c.bptr[j] + woff : zero_page;
            breg[j] = *(const u32x4*)p;
        }
        // advance by BK channels; when channels are a multiple of 64 this is uniform over the block
        c.ch += BK;
        if (uniform_tap) {
            if (c.ch >= a.Cs) {
                c.ch -= a.Cs;
                ++c.ltap;
                if (++c.tw >= c.ntw) { c.tw = 0; if (++c.th >= c.nth) { c.th = 0; ++c.kt; } }
            }
        } else {
            while (c.ch >= a.Cs) {
                c.ch -= a.Cs;
                ++c.ltap;
                if (++c.tw >= c.ntw) { c.tw = 0; if (++c.th >= c.nth) { c.th = 0; ++c.kt; } }
            }
        }
    };
    auto store_tiles = [&](int buf, const u32x4* areg, const u32x4* breg) {
        bf16_t* Ab = As + buf * BM * LDK;
        bf16_t* Bb = Bs + buf * BN * LDK;
#pragma unroll
        for (int i = 0; i < PA; ++i) *(u32x4*)(Ab + (i * RPP + lrow) * LDK + kvec * 8) = areg[i];
#pragma unroll
        for (int j = 0; j < PB; ++j) *(u32x4*)(Bb + (j * RPP + lrow) * LDK + kvec * 8) = breg[j];
    };

    int tile = next_tile(blockIdx.x);
    int rb = 0;
    Ctx ctx;
    if (tile >= 0) decode_rows(tile, 0);
    __syncthreads();   // also orders the zeroing of the statistics row
    if (tile >= 0) {
        ctx = make_ctx(tile, 0);
        load_tiles(ctx, areg, breg);
        if (PF2) load_tiles(ctx, areg1, breg1);
    }

    while (tile >= 0) {
        // The next tile's rows are decoded now and its first K step is fetched before this tile's
        // epilogue, so that the memory latency of a tile's first loads hides behind the previous epilogue.
        const int ntile = next_tile(tile + gridDim.x);
        if (ntile >= 0) decode_rows(ntile, rb ^ 1);

        f32x16 acc[MI][NJ];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        auto compute = [&](int buf) {
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
        };

        // Main loop.  The gathers of the next step (or next two steps, PF2) are in flight in registers while
        // the MFMAs of step k run out of LDS; LDS is double-buffered, one barrier per step.  On entry the
        // registers hold step 0 (and 1) of this tile.  Loads and LDS stores are issued unconditionally (steps
        // past the end read the zero page and land in a buffer nobody reads): with no branch around them the
        // compiler waits for exactly the older register set.
        const int nk = ctx.nk;
        store_tiles(0, areg, breg);
        __syncthreads();
        if (PF2) {
            for (int kc = 0; kc < nk; kc += 2) {
                load_tiles(ctx, areg, breg);
                compute(0);
                store_tiles(1, areg1, breg1);
                __syncthreads();
                if (kc + 1 >= nk) break;
                load_tiles(ctx, areg1, breg1);
                compute(1);
                store_tiles(0, areg, breg);
                __syncthreads();
            }
        } else {
            for (int kc = 0; kc < nk; ++kc) {
                const int buf = kc & 1;
                load_tiles(ctx, areg, breg);
                compute(buf);
                store_tiles(buf ^ 1, areg, breg);
                __syncthreads();
            }
        }
        const int n0 = ctx.n0;
        if (ntile >= 0) {
            ctx = make_ctx(ntile, rb ^ 1);
            load_tiles(ctx, areg, breg);
            if (PF2) load_tiles(ctx, areg1, breg1);
        }

        // ---- epilogue: round to bf16, per-channel statistics, stage through LDS, 16-byte stores.
        // D layout of the 32x32 MFMA: lane holds column (lane % 32); register r holds
        // row 8*(r/4) + 4*(lane/32) + r%4.  Neighbouring lanes swap one value of each row pair so
        // that every lane writes two adjacent columns of one row as a single 32-bit LDS store.
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            float s1 = 0.f, s2 = 0.f;
            const int col = wn * TN + j * 32 + (lane & 31);
            const bool odd = lane & 1;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float v0 = acc[i][j][r], v1 = acc[i][j][r + 1];
                    if (do_stats) {   // statistics of the values as stored (rows beyond M are exact zeros)
                        const uint32_t own = pack_bf16x2(v0, v1);
                        const float q0 = __uint_as_float(own << 16), q1 = __uint_as_float(own & 0xffff0000u);
                        s1 += q0 + q1;
                        s2 = fmaf(q0, q0, fmaf(q1, q1, s2));
                    }
                    const float got = __uint_as_float(pair_swap(__float_as_uint(odd ? v0 : v1)));
                    const uint32_t word = pack_bf16x2(odd ? got : v0, odd ? v1 : got);
                    const int row = wm * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3) + (odd ? 1 : 0);
                    *(uint32_t*)(Cst + row * LDC + (col & ~1)) = word;
                }
            }
            if (do_stats) {   // own slot: (wavefront row, lane half) x column
                const int slot = wm * 2 + (lane >> 5);
                s_part[slot * BN + col] = s1;
                s_part[(WM * 2 + slot) * BN + col] = s2;
            }
        }
        __syncthreads();
        if (do_stats && tid < 2 * BN) {   // fixed summation order over the slots, one thread per (statistic, column)
            const int stat = tid / BN, col = tid % BN;
            float v = 0.f;
#pragma unroll
            for (int sl = 0; sl < WM * 2; ++sl) v += s_part[(stat * WM * 2 + sl) * BN + col];
            if (n0 + col < a.Cd) atomicAdd(prow + stat * a.Cd + n0 + col, v);
        }
        {
            constexpr int CV = BN / 8;          // vectors per staged row
            constexpr int RPS = 256 / CV;       // rows per pass
            const int vcol = tid % CV, r0 = tid / CV;
            const int col = n0 + vcol * 8;
#pragma unroll
            for (int pss = 0; pss < BM / RPS; ++pss) {
                const int row = pss * RPS + r0;
                const int mrow = s_row[rb * BM + row].dst;
                if (mrow < 0 || col >= a.Cd) continue;
                const long m = mrow;
                u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
                if (!DGRAD) {
                    *(u32x4*)(a.dst + m * a.Cd + col) = v;
                } else {
                    const int dt = group_dt(col, a.fold);
                    auto emit = [&](long mr, bool with_value) {
                        u32x4 o = with_value ? v : u32x4{0u, 0u, 0u, 0u};
                        if (a.addend) {
                            const u32x4 ad = *(const u32x4*)(a.addend + mr * a.Cd + col);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const float lo = __uint_as_float(o[q] << 16) + __uint_as_float(ad[q] << 16);
                                const float hi = __uint_as_float(o[q] & 0xffff0000u) + __uint_as_float(ad[q] & 0xffff0000u);
                                o[q] = pack_bf16x2(lo, hi);
                            }
                        }
                        *(u32x4*)(a.dst + mr * a.Cd + col) = o;
                    };
                    if (dt == 0) {
                        emit(m, true);
                    } else {
                        const int t = (mrow / hw_d) % a.T;
                        if (t + dt >= 0 && t + dt < a.T) emit(m + (long)dt * hw_d, true);
                        // the frame that receives nothing from inside the clip
                        if ((dt == 1 && t == 0) || (dt == -1 && t == a.T - 1)) emit(m, false);
                    }
                }
            }
        }
        __syncthreads();
        tile = ntile;
        rb ^= 1;
    }

}

// ---------------------------------------------------------------------------------
// The same GEMM for source channel counts that are a multiple of 64 (every K step lies inside one tap), one
// block of WM*WN wavefronts per CU, a BM x BN tile.  What differs from igemm_kernel:
//
//  * Gathers are buffer loads: per tile every thread keeps one 32-bit byte offset per row it fetches; the part
//    of the address that changes from K step to K step (tap position, channel block) is the same for the whole
//    block and travels in the instruction's scalar offset, so a K step costs a mask test and a select per load
//    instead of 64-bit pointer arithmetic.  Lanes that fall on padding pass an offset beyond the buffer and
//    receive zeros from the bounds check.  The buffer starts `bias` bytes before the tensor so that the offset
//    of a row's tap origin, which may lie in the padding in front of the first frame, is never negative.
//  * LDS holds two stages.  A stage is the A rows [BM][64] followed by the B rows [BN][64], 128 bytes per row
//    without padding; position p (16 bytes) of row r holds the row's K vector p ^ ((r >> 1) & 7), which spreads
//    the 16-byte fragment reads of 16 consecutive rows over 16 different bank groups.  While step g is
//    multiplied out of one stage, step g+1 moves from registers into the other and step g+2 is loaded into the
//    registers, a few loads and stores after every group of MFMAs.  The stream of K steps runs across tile
//    boundaries, so a tile's first two steps are on the chip before the previous tile's epilogue starts.
static constexpr uint32_t OOB_OFFSET = 0x80000000u;   // buffers are smaller than 2 GiB

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

// CADD: the addend of a data gradient comes in the compact form described at IgemmArgs::add_stride (a variant of its
// own: the dense form stays free of the extra address arithmetic).
// MBITS: the ReLU decisions of a fused data-gradient epilogue come as one byte per eight channels (IgemmArgs::act_bits)
// instead of the activation itself: a sixteenth of the bytes.
template <int BM, int BN, int WM, int WN, bool DGRAD, bool STREAM, bool CADD = false, bool MBITS = false>
__global__ void __launch_bounds__(WM * WN * 64) igemm_ring_kernel(IgemmArgs a) {
    static_assert(DGRAD || !(CADD || MBITS), "only data gradients add a tensor or apply a mask");
    constexpr int NT = WM * WN * 64;                // threads
    constexpr int NS = 2;                           // LDS stages
    constexpr int MI = BM / (WM * 32), NJ = BN / (WN * 32);   // 32x32 MFMA tiles per wavefront
    constexpr int HM = BM / MI;                     // rows per epilogue pass; wavefront rows: i*HM + wm*32
    constexpr int TN = BN / WN;
    constexpr int KV = BK / 8;                      // 16-byte vectors per tile row
    constexpr int RPP = NT / KV;                    // tile rows loaded per pass
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int ROWB = BK * 2;                    // bytes per LDS row
    constexpr int STAGE = (BM + BN) * ROWB;         // bytes per ring stage
    constexpr int LDC = BN + 8;                     // staging pitch (elements)
    constexpr int NSLOT = WM * WN;                  // one statistics slot per wavefront
    static_assert(BK == 64 && KV == 8, "rows of eight 16-byte vectors");
    static_assert(BM % RPP == 0 && BN % RPP == 0 && HM == WM * 32, "tile / thread mismatch");
    static_assert((HM * LDC * 2) % 16 == 0, "alignment of the regions behind the staging tile");
    static_assert(sizeof(RowInfo) == 16, "one 16-byte LDS read per row");

    // 256-column tiles (forward, statistics epilogue only): the two stages take 128 KB, so the staging tile of the
    // epilogue lies in the stage that the tile's last K step was multiplied from.  Behind the barrier of that step no
    // wavefront reads it any more, and the next tile's steps are not written into it before the barrier at the top of
    // the next tile, which every wavefront reaches after its last read of the staging tile.
    constexpr bool ALIAS = BN == 256;
    static_assert(!ALIAS || (!DGRAD && HM * LDC * 2 <= STAGE), "the staging tile must fit a stage");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* Cst = (bf16_t*)(smem + NS * STAGE);      // [HM][LDC] staging tile of the epilogue (ALIAS: set per tile)
    float* s_part = ALIAS ? (float*)(smem + NS * STAGE) : (float*)(Cst + HM * LDC);   // [2 stats][WM*2 slots][BN] statistics slots
    RowInfo* s_row = (RowInfo*)(s_part + 2 * NSLOT * BN);   // [2][BM]: rows of the current and of the next tile
    int* s_arow = (int*)(s_row + 2 * BM);                   // [2][BM]: row of a compact addend (-1: none), dgrad only

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = tid / KV;                                   // row within a load pass
    const int kvec = (tid % KV) ^ ((lrow >> 1) & 7);             // K vector this thread fetches (see layout above)
    const bool do_stats = (!DGRAD) && a.stats != nullptr;
    const bool fuse_mask = DGRAD && (MBITS ? a.act_bits != nullptr : a.act != nullptr);   // ReLU mask in the epilogue ...
    const bool fuse_bn = fuse_mask && a.ybn != nullptr;      // ... and the BatchNorm-backward sums of the masked values

    const int hw_d = a.Hd * a.Wd;
    const int hw_s = a.Hs * a.Ws;
    const int frame_bytes = hw_s * a.pitch * 2;
    const int bias_el = (a.padh * a.Ws + a.padw) * a.pitch;      // the most negative tap origin, in elements
    const __amdgpu_buffer_rsrc_t rsrc_a =
        make_rsrc(a.src - bias_el, (uint32_t)(((long)a.F * hw_s * a.pitch + (a.Cs - a.pitch) + bias_el) * 2));
    const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(a.wp, (uint32_t)((long)a.Cd * a.K * 2));

    float* prow = (do_stats || fuse_bn) ? a.stats + (size_t)blockIdx.x * 2 * a.Cd : nullptr;
    if (do_stats || fuse_bn) {
        for (int c = tid; c < 2 * a.Cd; c += NT) prow[c] = 0.f;
    }

    const int mtiles = a.mt0[a.ncls];
    const int total_tiles = ((mtiles + 7) / 8) * 8 * a.ntiles;
    auto tile_mt = [&](int tile) { return ((tile >> 3) / a.ntiles) * 8 + (tile & 7); };
    auto next_tile = [&](int tile) {
        while (tile < total_tiles && tile_mt(tile) >= mtiles) tile += gridDim.x;
        return tile < total_tiles ? tile : -1;
    };

    // Producer view of one tile.  Everything but the per-row offsets and masks is the same for all threads.
    struct Ctx {
        int n0, nth, ntw, a0h, a0w, ntaps;
        int nk;               // K steps of the tile, at least two (steps beyond the data multiply zeros)
        uint32_t aoff[PA];    // byte offset of (row's tap origin, this thread's K vector) in the biased buffer
        uint32_t amask[PA];
        uint32_t boff[PB];    // byte offset of (output channel row, this thread's K vector) in the weights
        int kt, th, tw, chb, ltap;   // next K step to fetch: class-local tap, first channel of the step, flat tap
    };

    const bool pointwise = a.KT == 1 && a.KH == 1 && a.KW == 1 && a.stride == 1 && a.padh == 0 && a.padw == 0 && a.ncls == 1;
    auto decode_rows = [&](int tile, int rb) {
        if (tid < BM) {
            const int mt = tile_mt(tile);
            int cls = 0;
            while (cls + 1 < a.ncls && mt >= a.mt0[cls + 1]) ++cls;
            const int hc = a.hc[cls], wc = a.wc[cls];
            // (row counts are below 2^31: 32-bit divisions)
            const unsigned Mc = (unsigned)a.F * (unsigned)(hc * wc);
            const unsigned m = (unsigned)(mt - a.mt0[cls]) * BM + tid;
            RowInfo info;
            info.off = 0;
            info.mask = 0;
            info.dst = -1;
            if (m < Mc && pointwise) {
                // 1x1, stride 1: source row = destination row = m; only the shift needs the frame's place in its clip
                uint32_t mask = 1u | (1u << 8) | (1u << 30) | (1u << 31);
                if (a.fold > 0) {
                    const int t = (int)(m / (unsigned)hw_d) % a.T;
                    if (t + 1 >= a.T) mask &= ~(1u << 30);
                    if (t < 1) mask &= ~(1u << 31);
                }
                info.off = (long)m * a.pitch;
                info.mask = mask;
                info.dst = (int)m;
            } else if (m < Mc) {
                const int f = (int)(m / (unsigned)(hc * wc));
                const int q = (int)(m - (unsigned)f * (unsigned)(hc * wc));
                const int qh = (int)((unsigned)q / (unsigned)wc), qw = q - qh * wc;
                const int dh = qh * a.cstep + a.ph[cls], dw = qw * a.cstep + a.pw[cls];
                // (the class step is 1 or 2 and divides the numerators exactly, negative ones included)
                const int sh = a.cstep == 2 ? 1 : 0;
                const int oh = DGRAD ? (dh - a.padh + a.a0h[cls]) >> sh : dh * a.stride - a.padh;
                const int ow = DGRAD ? (dw - a.padw + a.a0w[cls]) >> sh : dw * a.stride - a.padw;
                const int t = f % a.T;
                uint32_t mask = 0;
                for (int th = 0; th < a.nth[cls]; ++th)
                    if (oh + th >= 0 && oh + th < a.Hs) mask |= 1u << th;
                for (int tw = 0; tw < a.ntw[cls]; ++tw)
                    if (ow + tw >= 0 && ow + tw < a.Ws) mask |= 1u << (8 + tw);
                if (t + 1 < a.T) mask |= 1u << 30;
                if (t >= 1) mask |= 1u << 31;
                info.off = ((long)f * hw_s + (long)oh * a.Ws + ow) * a.pitch;
                info.mask = mask;
                info.dst = (f * a.Hd + dh) * a.Wd + dw;
            }
            s_row[rb * BM + tid] = info;
            if (CADD) {
                // the destination pixel's place in the compact addend (frame offsets of the adjoint shift are added
                // where the row is used: they do not change the pixel)
                int arow = -1;
                if (info.dst >= 0) {
                    const unsigned f = (unsigned)info.dst / (unsigned)hw_d, q = (unsigned)info.dst - f * (unsigned)hw_d;
                    const unsigned h = q / (unsigned)a.Wd, w = q - h * (unsigned)a.Wd;
                    if (((h | w) & 1u) == 0) arow = (int)((f * (unsigned)a.add_ho + (h >> 1)) * (unsigned)a.add_wo + (w >> 1));
                }
                s_arow[rb * BM + tid] = arow;
            }
        }
    };
    auto make_ctx = [&](int tile, int rb) {
        Ctx c;
        const int mt = tile_mt(tile);
        int cls = 0;
        while (cls + 1 < a.ncls && mt >= a.mt0[cls + 1]) ++cls;
        c.n0 = ((tile >> 3) % a.ntiles) * BN;
        c.nth = a.nth[cls]; c.ntw = a.ntw[cls]; c.a0h = a.a0h[cls]; c.a0w = a.a0w[cls];
        c.ntaps = a.KT * c.nth * c.ntw;
        c.nk = c.ntaps * (a.Cs / BK);
        if (c.nk < 2) c.nk = 2;
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const RowInfo ri = s_row[rb * BM + i * RPP + lrow];
            c.aoff[i] = (uint32_t)((ri.off + bias_el) * 2) + kvec * 16;
            c.amask[i] = ri.mask;
        }
#pragma unroll
        for (int j = 0; j < PB; ++j) {
            const int n = c.n0 + j * RPP + lrow;
            c.boff[j] = n < a.Cd ? (uint32_t)n * (uint32_t)a.K * 2u + kvec * 16 : OOB_OFFSET;
        }
        c.kt = c.th = c.tw = c.ltap = c.chb = 0;
        return c;
    };

    // The gathers of one K step: per-thread offsets (OOB_OFFSET for padding), block-wide scalar offsets.
    constexpr int NP = PA + PB;
    struct Plan {
        uint32_t v[NP];
        int soff_a, soff_b;
    };
    // Plans the producer's next K step and advances its position.  `live` false: nothing is left to fetch and
    // the step is all zeros.
    auto plan = [&](Ctx& c, bool live) {
        Plan p;
        const bool kvalid = live && c.ltap < c.ntaps;
        const int d0 = c.kt - a.KT / 2;                              // frame offset of a temporal tap
        const bool lane_dt = !DGRAD && a.fold > 0 && c.chb < 2 * a.fold;   // shifted channels in this step
        const uint32_t need0 = (1u << c.th) | (1u << (8 + c.tw));
        p.soff_a = ((c.th * a.Ws + c.tw) * a.pitch + c.chb) * 2;
        const int ta = c.a0h + c.th * a.cstep, tb = c.a0w + c.tw * a.cstep;   // (flipped) tap coordinates
        p.soff_b = (((c.kt * a.KH + ta) * a.KW + tb) * a.Cs + c.chb) * 2;
        if (!kvalid) {
            p.soff_a = p.soff_b = 0;
#pragma unroll
            for (int i = 0; i < NP; ++i) p.v[i] = OOB_OFFSET;
        } else {
            if (!lane_dt && d0 == 0) {
#pragma unroll
                for (int i = 0; i < PA; ++i) p.v[i] = (c.amask[i] & need0) == need0 ? c.aoff[i] : OOB_OFFSET;
            } else {
                const int d = d0 + (lane_dt ? group_dt(c.chb + kvec * 8, a.fold) : 0);   // in {-1, 0, 1}
                const uint32_t need = need0 | (d > 0 ? 1u << 30 : 0u) | (d < 0 ? 1u << 31 : 0u);
                const int dl = d * frame_bytes;
#pragma unroll
                for (int i = 0; i < PA; ++i) p.v[i] = (c.amask[i] & need) == need ? c.aoff[i] + (uint32_t)dl : OOB_OFFSET;
            }
#pragma unroll
            for (int j = 0; j < PB; ++j) p.v[PA + j] = c.boff[j];
        }
        c.chb += BK;
        if (c.chb >= a.Cs) {
            c.chb = 0;
            ++c.ltap;
            if (++c.tw >= c.ntw) { c.tw = 0; if (++c.th >= c.nth) { c.th = 0; ++c.kt; } }
        }
        return p;
    };
    // One 16-byte piece of a K step per call: pieces 0..PA-1 are A rows, the rest B rows.  A piece is loaded
    // into its register during one step and written to the ring during the next one.
    u32x4 greg[NP];
    auto load_piece = [&](const Plan& p, int i) {
        greg[i] = i < PA ? __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, (int)p.v[i], p.soff_a, 0)
                         : __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, (int)p.v[i], p.soff_b, 0);
    };
    auto store_piece = [&](int stage, int i) {   // thread -> row lrow of the piece's pass, position tid % 8
        const int row0 = i < PA ? i * RPP : BM + (i - PA) * RPP;
        *(u32x4*)(smem + stage * STAGE + row0 * ROWB + tid * 16) = greg[i];
    };

    // fragment addresses inside a stage: row (lane % 32) of the wavefront's first row block, K vector
    // 2*ks + lane/32 at its swizzled position
    int a_rd[BK / 16], b_rd[BK / 16];
    {
        const int r = lane & 31, hi = lane >> 5, sw = (r >> 1) & 7;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int pos = ((2 * ks + hi) ^ sw) * 16;
            a_rd[ks] = (wm * 32 + r) * ROWB + pos;
            b_rd[ks] = (BM + wn * TN + r) * ROWB + pos;
        }
    }

    int tile = next_tile(blockIdx.x);
    int rb = 0;
    int cstage = 0;                  // stage being multiplied; the other one is being filled
    Ctx pc;                          // producer position
    int p_left = 0;                  // K steps the producer still has to fetch for its tile
    bool p_on_next = false;          // the producer has moved on to the tile after the current one
    if (tile >= 0) decode_rows(tile, 0);
    __syncthreads();                 // also orders the zeroing of the statistics row
    if (tile >= 0) {
        pc = make_ctx(tile, 0);
        p_left = pc.nk - 2;
        Plan p0 = plan(pc, true);
#pragma unroll
        for (int i = 0; i < NP; ++i) load_piece(p0, i);
#pragma unroll
        for (int i = 0; i < NP; ++i) store_piece(0, i);
        Plan p1 = plan(pc, true);
#pragma unroll
        for (int i = 0; i < NP; ++i) load_piece(p1, i);
    }
    int cur_nk = tile >= 0 ? pc.nk : 0, cur_n0 = tile >= 0 ? pc.n0 : 0;
    // Fragment registers live across K steps and tiles: the first fragments of a step are read from its stage
    // while the last MFMA group of the step before is still in the pipeline (see the main loop).
    constexpr int KS = BK / 16;
    bf16x8 af[2][MI], bfr[2][NJ];
    __syncthreads();                 // stage 0 holds the first step
#pragma unroll
    for (int i = 0; i < MI; ++i) af[0][i] = *(const bf16x8*)(smem + a_rd[0] + i * HM * ROWB);
#pragma unroll
    for (int j = 0; j < NJ; ++j) bfr[0][j] = *(const bf16x8*)(smem + b_rd[0] + j * 32 * ROWB);
    // Per-channel sums (forward statistics, or the BatchNorm-backward sums of a fused data gradient) of the eight
    // columns this thread stores.  They run on across the tiles of the block as long as the column tile stays the
    // same (with a grid that is a multiple of 8 * ntiles it never changes) and are reduced and flushed when it
    // changes and after the last tile.
    constexpr int FV = 8;
    float f1[FV], f2[FV];
#pragma unroll
    for (int q = 0; q < FV; ++q) f1[q] = f2[q] = 0.f;

    while (tile >= 0) {
        const int ntile = next_tile(tile + gridDim.x);
        if (ntile >= 0) decode_rows(ntile, rb ^ 1);   // published by the first barrier of the main loop

        f32x16 acc[MI][NJ];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        // Main loop.  On entry to step g (stream position of the block, across tiles) stage g % 2 holds step g
        // and the registers hold step g+1, loaded during step g-1.  While step g is multiplied, the registers
        // are written to the other stage piece by piece and each freed register is reloaded with its piece of
        // step g+2.  The pieces are spread over the MFMA groups: issued in one burst, the loads of all eight
        // wavefronts would fill the address unit's queue and stall the wavefronts in front of their MFMAs.
        int next_nk = 0, next_n0 = 0;
        // Plans the step the producer fetches next; the producer crosses into the next tile when it has
        // fetched all steps of its tile.
        auto plan_next = [&]() {
            if (p_left == 0 && !p_on_next) {
                p_on_next = true;
                if (ntile >= 0) {
                    pc = make_ctx(ntile, rb ^ 1);
                    p_left = pc.nk;
                    next_nk = pc.nk;
                    next_n0 = pc.n0;
                }
            }
            const bool live = p_left > 0;
            if (live) --p_left;
            return plan(pc, live);
        };
        __syncthreads();       // the next tile's rows are decoded
        Plan pl = plan_next();
        for (int kc = 0; kc < cur_nk; ++kc) {
            // One barrier per step, in front of the last MFMA group: by then every wavefront has written its pieces
            // of the next step into the other stage and has read its last fragments of this stage, so behind the
            // barrier the next step's first fragments are read (their latency overlaps the last MFMA group) and
            // the next step may overwrite this stage.
            const unsigned char* st = smem + cstage * STAGE;
            const unsigned char* stn = smem + (cstage ^ 1) * STAGE;
            constexpr int PPK = (NP + KS - 2) / (KS - 1);     // pieces handled after each of the first KS-1 groups
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int cb = ks & 1, nb = cb ^ 1;
                if (ks + 1 < KS) {
#pragma unroll
                    for (int i = 0; i < MI; ++i) af[nb][i] = *(const bf16x8*)(st + a_rd[ks + 1] + i * HM * ROWB);
#pragma unroll
                    for (int j = 0; j < NJ; ++j) bfr[nb][j] = *(const bf16x8*)(st + b_rd[ks + 1] + j * 32 * ROWB);
                } else {
                    __syncthreads();
#pragma unroll
                    for (int i = 0; i < MI; ++i) af[nb][i] = *(const bf16x8*)(stn + a_rd[0] + i * HM * ROWB);
#pragma unroll
                    for (int j = 0; j < NJ; ++j) bfr[nb][j] = *(const bf16x8*)(stn + b_rd[0] + j * 32 * ROWB);
                }
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        // operands swapped: the result block is [channel][pixel], so a lane holds four consecutive
                        // channels of one pixel per register quad, which the epilogue stores to LDS as one 8-byte piece
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cb][j], af[cb][i], acc[i][j], 0, 0, 0);
#pragma unroll
                for (int q = ks * PPK; q < (ks + 1) * PPK && q < NP; ++q) {
                    store_piece(cstage ^ 1, q);
                    load_piece(pl, q);
                }
                __builtin_amdgcn_sched_barrier(0);   // keep the pieces where they are
            }
            // the address arithmetic of the next step runs while the last MFMAs of this one are in the pipeline
            if (kc + 1 < cur_nk) pl = plan_next();
            cstage ^= 1;
        }

        // ---- epilogue, one pass per row block through the staging tile; the registers and the other LDS
        // stage already hold the first two K steps of the next tile.
        // fused BatchNorm backward: this thread stores the same eight columns of every row it handles
        // (forward with an affine epilogue keeps scale / shift of the same eight columns in mu / rs)
        if (ALIAS) Cst = (bf16_t*)(smem + (cstage ^ 1) * STAGE);
        const bool affine = !DGRAD && !ALIAS && a.ep_scale != nullptr;
        float mu[FV], rs[FV];
#pragma unroll
        for (int q = 0; q < FV; ++q) mu[q] = rs[q] = 0.f;
        if (fuse_bn || affine) {
            const int c0 = cur_n0 + (tid % (BN / 8)) * 8;
            if (c0 < a.Cd) {
#pragma unroll
                for (int q = 0; q < FV; ++q) {
                    mu[q] = DGRAD ? a.bn_mean[c0 + q] : a.ep_scale[c0 + q];
                    rs[q] = DGRAD ? a.bn_rstd[c0 + q] : a.ep_shift[c0 + q];
                }
            }
        }
        // Data gradient: addend, ReLU mask source and BatchNorm input of a pass are requested before the
        // barriers and the staging of that pass, so that their latency overlaps them.  A row's value goes to
        // frame t + dt of its channel group (adjoint shift); the frame of the group that receives nothing from
        // inside the clip gets a zero value (rare, handled after the regular rows).
        constexpr int CV = BN / 8;          // vectors per staged row
        constexpr int RPS = NT / CV;        // rows per pass of the store loop
        constexpr int NPS = HM / RPS;
        constexpr int NPD = DGRAD ? NPS : 1;
        const int vcol = tid % CV, r0 = tid / CV;
        const int col = cur_n0 + vcol * 8;
        long mr[NPD], mz[NPD];
        u32x4 ad[NPD], ac[NPD], yy[NPD];
        const bf16_t* zero_page_d = (const bf16_t*)g_zero_page;
        auto request = [&](int h) {
            const int dt = group_dt(col, a.fold);
#pragma unroll
            for (int pss = 0; pss < NPD; ++pss) {
                const int mrow = s_row[rb * BM + h * HM + pss * RPS + r0].dst;
                const bool live = mrow >= 0 && col < a.Cd;
                const int t = live ? (mrow / hw_d) % a.T : 0;
                const bool in_clip = t + dt >= 0 && t + dt < a.T;
                mr[pss] = live && in_clip ? (long)mrow + (long)dt * hw_d : -1;
                mz[pss] = live && ((dt == 1 && t == 0) || (dt == -1 && t == a.T - 1)) ? mrow : -1;
                // loads without a branch around them (rows that are not stored read the zero page): a load
                // under a condition would be awaited where the branches join
                const long e = mr[pss] * a.Cd + col;
                const bool ok = mr[pss] >= 0;
                if (CADD) {
                    const int arow = s_arow[rb * BM + h * HM + pss * RPS + r0];
                    const long ea = ((long)arow + (long)dt * (a.add_ho * a.add_wo)) * a.Cd + col;
                    ad[pss] = *(const u32x4*)((ok && arow >= 0) ? a.addend + ea : zero_page_d);
                } else {
                    ad[pss] = *(const u32x4*)((ok && a.addend) ? a.addend + e : zero_page_d);
                }
                if (MBITS) {
                    // (bit j of the byte: channel col + j; rows that are not stored read a zero byte)
                    ac[pss][0] = *((ok && fuse_mask) ? a.act_bits + (mr[pss] * a.Cd + col) / 8 : (const uint8_t*)zero_page_d);
                } else {
                    ac[pss] = *(const u32x4*)((ok && fuse_mask) ? a.act + e : zero_page_d);
                }
                yy[pss] = *(const u32x4*)((ok && fuse_bn) ? a.ybn + e : zero_page_d);
            }
        };
        if (DGRAD) request(0);
#pragma unroll
        for (int h = 0; h < MI; ++h) {
            if (h > 0) __syncthreads();   // previous pass stored (the previous tile's last pass: barrier at its end)
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                // lane: pixel lane % 32 of the row block, channels 8*q + 4*(lane / 32) + {0..3} of the column block
                bf16_t* dstp = Cst + (wm * 32 + (lane & 31)) * LDC + wn * TN + j * 32 + 4 * (lane >> 5);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 w;
                    w.x = pack_bf16x2(acc[h][j][4 * q], acc[h][j][4 * q + 1]);
                    w.y = pack_bf16x2(acc[h][j][4 * q + 2], acc[h][j][4 * q + 3]);
                    *(uint2*)(dstp + 8 * q) = w;
                }
            }
            __syncthreads();
            if (!DGRAD) {
#pragma unroll
                for (int pss = 0; pss < HM / RPS; ++pss) {
                    const int row = pss * RPS + r0;
                    const int mrow = s_row[rb * BM + h * HM + row].dst;
                    if (mrow < 0 || col >= a.Cd) continue;
                    u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
                    u32x4* q = (u32x4*)(a.dst + (long)mrow * a.Cd + col);
                    if (do_stats) {   // statistics of the values as stored
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float lo = __uint_as_float(v[e] << 16), hi = __uint_as_float(v[e] & 0xffff0000u);
                            f1[2 * e] += lo;
                            f1[2 * e + 1] += hi;
                            f2[2 * e] = fmaf(lo, lo, f2[2 * e]);
                            f2[2 * e + 1] = fmaf(hi, hi, f2[2 * e + 1]);
                        }
                    }
                    if (affine) {
                        u32x4 r = u32x4{0u, 0u, 0u, 0u};
                        if (a.ep_res) r = *(const u32x4*)(a.ep_res + (long)mrow * a.Cd + col);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float lo = fmaf(__uint_as_float(v[e] << 16), mu[2 * e], rs[2 * e]) + __uint_as_float(r[e] << 16);
                            float hi = fmaf(__uint_as_float(v[e] & 0xffff0000u), mu[2 * e + 1], rs[2 * e + 1]) + __uint_as_float(r[e] & 0xffff0000u);
                            if (a.ep_relu) {
                                lo = lo > 0.f ? lo : 0.f;
                                hi = hi > 0.f ? hi : 0.f;
                            }
                            v[e] = pack_bf16x2(lo, hi);
                        }
                    }
                    if (STREAM) __builtin_nontemporal_store(v, q);
                    else *q = v;
                }
            } else {
                // value (+ addend) -> optional ReLU mask and BatchNorm sums -> store
                auto finish = [&](long mr, u32x4 o, const u32x4& ad, const u32x4& ac, const u32x4& yy) {
                    if (a.addend) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float lo = __uint_as_float(o[q] << 16) + __uint_as_float(ad[q] << 16);
                            const float hi = __uint_as_float(o[q] & 0xffff0000u) + __uint_as_float(ad[q] & 0xffff0000u);
                            o[q] = pack_bf16x2(lo, hi);
                        }
                    }
                    if (fuse_mask) {   // on the values as stored (bf16); without ybn the sums are not used
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const bool plo = MBITS ? ((ac[0] >> (2 * q)) & 1u) != 0 : __uint_as_float(ac[q] << 16) > 0.f;
                            const bool phi = MBITS ? ((ac[0] >> (2 * q + 1)) & 1u) != 0 : __uint_as_float(ac[q] & 0xffff0000u) > 0.f;
                            const float dlo = plo ? __uint_as_float(o[q] << 16) : 0.f;
                            const float dhi = phi ? __uint_as_float(o[q] & 0xffff0000u) : 0.f;
                            o[q] = (plo ? o[q] & 0xffffu : 0u) | (phi ? o[q] & 0xffff0000u : 0u);
                            f1[2 * q] += dlo;
                            f1[2 * q + 1] += dhi;
                            f2[2 * q] = fmaf(dlo, (__uint_as_float(yy[q] << 16) - mu[2 * q]) * rs[2 * q], f2[2 * q]);
                            f2[2 * q + 1] = fmaf(dhi, (__uint_as_float(yy[q] & 0xffff0000u) - mu[2 * q + 1]) * rs[2 * q + 1], f2[2 * q + 1]);
                        }
                    }
                    u32x4* q = (u32x4*)(a.dst + mr * a.Cd + col);
                    if (STREAM) __builtin_nontemporal_store(o, q);
                    else *q = o;
                };
#pragma unroll
                for (int pss = 0; pss < NPS; ++pss)
                    if (mr[pss] >= 0) finish(mr[pss], *(const u32x4*)(Cst + (pss * RPS + r0) * LDC + vcol * 8), ad[pss], ac[pss], yy[pss]);
#pragma unroll
                for (int pss = 0; pss < NPS; ++pss) {
                    if (mz[pss] < 0) continue;
                    const long e = mz[pss] * a.Cd + col;
                    u32x4 zad = u32x4{0u, 0u, 0u, 0u}, zac = zad, zyy = zad;
                    if (CADD) {
                        const int arow = s_arow[rb * BM + h * HM + pss * RPS + r0];
                        if (arow >= 0) zad = *(const u32x4*)(a.addend + (long)arow * a.Cd + col);
                    } else if (a.addend) {
                        zad = *(const u32x4*)(a.addend + e);
                    }
                    if (fuse_mask) {
                        if (MBITS) zac[0] = a.act_bits[e / 8];
                        else zac = *(const u32x4*)(a.act + e);
                    }
                    if (fuse_bn) zyy = *(const u32x4*)(a.ybn + e);
                    finish(mz[pss], u32x4{0u, 0u, 0u, 0u}, zad, zac, zyy);
                }
                if (h + 1 < MI) request(h + 1);
            }
        }
        if ((fuse_bn || do_stats) && (ntile < 0 || next_n0 != cur_n0)) {
            // lanes CV apart hold the same columns: fold them, then one slot per wavefront, fixed order over the slots
            constexpr int CV = BN / 8;
#pragma unroll
            for (int q = 0; q < FV; ++q) {
#pragma unroll
                for (int off = CV; off < 64; off <<= 1) {
                    f1[q] += __shfl_xor(f1[q], off);
                    f2[q] += __shfl_xor(f2[q], off);
                }
            }
            if (lane < CV) {
#pragma unroll
                for (int q = 0; q < FV; ++q) {
                    s_part[wave * BN + lane * 8 + q] = f1[q];
                    s_part[(NSLOT + wave) * BN + lane * 8 + q] = f2[q];
                }
            }
            __syncthreads();
            if (tid < 2 * BN) {
                const int stat = tid / BN, col = tid % BN;
                float v = 0.f;
#pragma unroll
                for (int sl = 0; sl < NSLOT; ++sl) v += s_part[(stat * NSLOT + sl) * BN + col];
                if (cur_n0 + col < a.Cd) atomicAdd(prow + stat * a.Cd + cur_n0 + col, v);
            }
#pragma unroll
            for (int q = 0; q < FV; ++q) f1[q] = f2[q] = 0.f;
        }
        __syncthreads();   // the row buffer of this tile is decoded into again at the top of the next tile
        tile = ntile;
        rb ^= 1;
        cur_nk = next_nk;
        cur_n0 = next_n0;
        p_on_next = false;
    }
}

// ---------------------------------------------------------------------------------
// 3x3, stride 1, pad 1, 64 -> 64 channels, no shift: the middle convolution of the first stage (and its data
// gradient, which is the same convolution with the flipped, transposed weights).  These layers have the most
// pixels per FLOP of all 3x3 layers (56x56 maps) and K = 576 is only nine steps, so in the general kernel above
// they pay nine gathers of the input and a barrier per 16 MFMAs.  Here everything a tile needs sits in LDS:
//
//  * the weights of all nine taps (72 KB), loaded once per block and kept for all of its tiles;
//  * the tile's input patch: the 256 pixels of the tile are consecutive rows of the [pixel][64] tensor, and
//    the neighbours (h + th - 1, w + tw - 1) of pixel p are rows p + (th - 1) * W + (tw - 1), so the patch is
//    the row range [p0 - W - 1, p0 + 256 + W + 1), read from memory once.  A tap is then a row offset into the
//    patch, the same for every lane; the lanes whose neighbour lies outside the frame read a row of zeros
//    instead (one select on the address per tap, no select on the data);
//  * patch rows are 144 bytes apart (128 + 16): the rows of 16 consecutive pixels then fall 36 banks apart and
//    a fragment read is conflict-free at every tap offset, which a swizzle tied to the row number is not.
//
// The main loop of a tile has no barrier and no global load of its own: while it runs, the next tile's patch
// is fetched into registers (six 16-byte pieces per thread) and written to LDS after the last MFMA.
static constexpr int C64_BM = 256;                            // pixels per tile
static constexpr int C64_WMAX = 57;                           // widest map: the patch has BM + 2 * (W + 1) rows
static constexpr int C64_PROW = 144;                          // bytes per patch row
static constexpr int C64_PR = C64_BM + 2 * (C64_WMAX + 1);    // patch rows at the widest map
static constexpr int C64_NPP = (C64_PR * 8 + 511) / 512;      // 16-byte patch pieces per thread
static constexpr int C64_W_BYTES = 9 * 64 * 128;
static constexpr int C64_PATCH_BYTES = C64_PR * C64_PROW;
static constexpr int C64_ZERO_BYTES = 160;                    // a fragment's reach from the zero row: 16 + 3 * 32 + 16
static constexpr int C64_LDC = 64 + 8;                        // staging pitch (elements)
static constexpr int C64_CST_BYTES = 128 * C64_LDC * 2;
static constexpr int C64_PART_BYTES = 2 * 8 * 64 * 4;
static constexpr int C64_SMEM = C64_W_BYTES + C64_PATCH_BYTES + C64_ZERO_BYTES + C64_CST_BYTES + C64_PART_BYTES;
static_assert(C64_SMEM <= 160 * 1024, "LDS budget");
static_assert(C64_PATCH_BYTES % 16 == 0 && C64_ZERO_BYTES % 16 == 0 && C64_CST_BYTES % 16 == 0, "alignment");

template <bool DGRAD, bool STREAM>
__global__ void __launch_bounds__(512) conv3x3_c64_kernel(IgemmArgs a) {
    constexpr int NT = 512, BM = C64_BM, BN = 64, MI = 2, HM = 128, LDC = C64_LDC, PROW = C64_PROW, NPP = C64_NPP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;                                    // [9][64][8 positions of 16 bytes], swizzled
    unsigned char* s_patch = smem + C64_W_BYTES;                  // [patch rows][144 bytes]
    constexpr int ZERO_OFF = C64_PATCH_BYTES;                     // the zero row, as an offset from s_patch
    bf16_t* Cst = (bf16_t*)(s_patch + C64_PATCH_BYTES + C64_ZERO_BYTES);   // [128][LDC] staging tile of the epilogue
    float* s_part = (float*)((unsigned char*)Cst + C64_CST_BYTES);         // [2 stats][8 wavefronts][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;        // wavefront: rows wm*32 (+128 for the second row block), channels wn*32
    const int r = lane & 31, hi = lane >> 5;
    const int W = a.Ws, H = a.Hs, hw = H * W;
    const unsigned M = (unsigned)a.F * (unsigned)hw;              // pixels (source and destination maps coincide)
    const int mtiles = (int)((M + BM - 1) / BM);
    const bool do_stats = !DGRAD && a.stats != nullptr;
    const bool fuse_mask = DGRAD && a.act != nullptr;
    const bool fuse_bn = fuse_mask && a.ybn != nullptr;
    const bool affine = !DGRAD && a.ep_scale != nullptr;

    float* prow = (do_stats || fuse_bn) ? a.stats + (size_t)blockIdx.x * 2 * BN : nullptr;
    if (prow && tid < 2 * BN) prow[tid] = 0.f;

    // ---- weights and the zero row
    {
        const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(a.wp, (uint32_t)(BN * 9 * 64 * 2));
#pragma unroll
        for (int s = 0; s < 9; ++s) {
            const int q = tid + s * NT;                           // piece: tap s, channel row n, position pos
            const int n = (q >> 3) & 63, pos = q & 7, kv = pos ^ ((n >> 1) & 7);
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, n * (9 * 128) + s * 128 + kv * 16, 0, 0);
            *(u32x4*)(s_w + q * 16) = v;
        }
        if (tid < C64_ZERO_BYTES / 16) *(u32x4*)(s_patch + ZERO_OFF + tid * 16) = u32x4{0u, 0u, 0u, 0u};
    }

    // ---- the patch producer.  Row j of the patch is row p0 + j of the buffer, which starts W + 1 rows before
    // the tensor (rows in front of the tensor and behind its end are never fetched: they read as zeros).
    const int lead = W + 1;
    const int npieces = (BM + 2 * lead) * 8;
    const __amdgpu_buffer_rsrc_t rsrc_a =
        make_rsrc(a.src - (long)lead * 64, (uint32_t)(((long)M + lead) * 128));
    u32x4 preg[NPP];
    auto load_patch = [&](int tile) {
        const unsigned p0 = (unsigned)tile * BM;
#pragma unroll
        for (int s = 0; s < NPP; ++s) {
            const int q = tid + s * NT;
            const unsigned row = p0 + (unsigned)(q >> 3);
            const bool ok = q < npieces && row >= (unsigned)lead;
            preg[s] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, ok ? (int)(row * 128u + (unsigned)(q & 7) * 16u) : (int)OOB_OFFSET, 0, 0);
        }
    };
    auto store_patch = [&]() {
#pragma unroll
        for (int s = 0; s < NPP; ++s) {
            const int q = tid + s * NT;
            if (q < npieces) *(u32x4*)(s_patch + (q >> 3) * PROW + (q & 7) * 16) = preg[s];
        }
    };

    // ---- fragment addresses: weights row (lane % 32) of the wavefront's channel block, K vector 2*ks + lane/32 at
    // its swizzled position; patch row (lane % 32) of the wavefront's row block (tap offset added per tap)
    int b_rd[4], a_base[MI];
    {
        const int n = wn * 32 + r;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) b_rd[ks] = n * 128 + (((2 * ks + hi) ^ ((n >> 1) & 7)) * 16);
#pragma unroll
        for (int i = 0; i < MI; ++i) a_base[i] = (i * HM + wm * 32 + r) * PROW + hi * 16;
    }
    const int zero_addr = ZERO_OFF + hi * 16;

    constexpr int FV = 8, CV = BN / 8, RPS = NT / CV, NPS = HM / RPS;
    float f1[FV], f2[FV];
#pragma unroll
    for (int q = 0; q < FV; ++q) f1[q] = f2[q] = 0.f;
    const int vcol = tid % CV, r0 = tid / CV;
    // the eight channels this thread stores: BatchNorm mean / rstd of a fused data gradient, or scale / shift of an
    // affine forward epilogue
    float mu[FV], rs[FV];
#pragma unroll
    for (int q = 0; q < FV; ++q) mu[q] = rs[q] = 0.f;
    if (fuse_bn || affine) {
#pragma unroll
        for (int q = 0; q < FV; ++q) {
            mu[q] = DGRAD ? a.bn_mean[vcol * 8 + q] : a.ep_scale[vcol * 8 + q];
            rs[q] = DGRAD ? a.bn_rstd[vcol * 8 + q] : a.ep_shift[vcol * 8 + q];
        }
    }

    // Blocks are dealt round-robin over the eight XCDs, each with an L2 of its own: an XCD takes a contiguous eighth
    // of the tiles, so that the patch rows a tile shares with its neighbours are found in that L2.
    const bool by_xcd = (gridDim.x % 8) == 0;
    const int per_xcd = by_xcd ? (mtiles + 7) / 8 : mtiles;
    const int xcd = by_xcd ? (int)(blockIdx.x % 8) : 0;
    const int seq_step = by_xcd ? (int)(gridDim.x / 8) : (int)gridDim.x;
    auto tile_at = [&](int seq) {
        const int t = xcd * per_xcd + seq;
        return (seq < per_xcd && t < mtiles) ? t : -1;
    };
    int seq = by_xcd ? (int)(blockIdx.x / 8) : (int)blockIdx.x;
    int tile = tile_at(seq);
    if (tile >= 0) load_patch(tile);
    __syncthreads();                      // weights, zero row, statistics row
    if (tile >= 0) store_patch();

    while (tile >= 0) {
        seq += seq_step;
        const int ntile = tile_at(seq);
        __syncthreads();                  // this tile's patch is in LDS

        // which of the nine neighbours of this lane's pixels lie inside the frame (bit th*3 + tw)
        unsigned vmask[MI];
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const unsigned P = (unsigned)tile * BM + (unsigned)(i * HM + wm * 32 + r);
            unsigned m = 0;
            if (P < M) {
                const int q = (int)(P % (unsigned)hw);
                const int h = q / W, w = q - h * W;
                const unsigned rows_ok = (h > 0 ? 1u : 0u) | 2u | (h + 1 < H ? 4u : 0u);
                const unsigned cols_ok = (w > 0 ? 1u : 0u) | 2u | (w + 1 < W ? 4u : 0u);
#pragma unroll
                for (int th = 0; th < 3; ++th)
                    if (rows_ok >> th & 1u) m |= cols_ok << (3 * th);
            }
            vmask[i] = m;
        }

        f32x16 acc[MI];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

        if (ntile >= 0) load_patch(ntile);   // lands in registers while this tile is multiplied

#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
            const int toff = ((tap / 3) * W + (tap % 3)) * PROW;
            int a_addr[MI];
#pragma unroll
            for (int i = 0; i < MI; ++i) a_addr[i] = (vmask[i] >> tap & 1u) ? a_base[i] + toff : zero_addr;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 bfr = *(const bf16x8*)(s_w + tap * (64 * 128) + b_rd[ks]);
                bf16x8 af[MI];
#pragma unroll
                for (int i = 0; i < MI; ++i) af[i] = *(const bf16x8*)(s_patch + a_addr[i] + ks * 32);
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    // operands swapped as in igemm_ring_kernel: the result block is [channel][pixel]
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af[i], acc[i], 0, 0, 0);
            }
        }

        __syncthreads();                  // every wavefront has read its last fragment of the patch
        if (ntile >= 0) store_patch();

        // ---- epilogue, one pass per row block through the staging tile
#pragma unroll
        for (int h = 0; h < MI; ++h) {
            if (h > 0) __syncthreads();
            {
                // lane: pixel lane % 32 of the wavefront's rows, channels 8*q + 4*(lane / 32) + {0..3} of its channel block
                bf16_t* dstp = Cst + (wm * 32 + r) * LDC + wn * 32 + 4 * hi;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 w2;
                    w2.x = pack_bf16x2(acc[h][4 * q], acc[h][4 * q + 1]);
                    w2.y = pack_bf16x2(acc[h][4 * q + 2], acc[h][4 * q + 3]);
                    *(uint2*)(dstp + 8 * q) = w2;
                }
            }
            __syncthreads();
#pragma unroll
            for (int pss = 0; pss < NPS; ++pss) {
                const int row = pss * RPS + r0;
                const unsigned P = (unsigned)tile * BM + (unsigned)(h * HM + row);
                if (P >= M) continue;
                u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
                const long e = (long)P * BN + vcol * 8;
                if (!DGRAD) {
                    if (do_stats) {   // statistics of the values as stored
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float lo = __uint_as_float(v[q] << 16), hi2 = __uint_as_float(v[q] & 0xffff0000u);
                            f1[2 * q] += lo;
                            f1[2 * q + 1] += hi2;
                            f2[2 * q] = fmaf(lo, lo, f2[2 * q]);
                            f2[2 * q + 1] = fmaf(hi2, hi2, f2[2 * q + 1]);
                        }
                    }
                    if (affine) {
                        u32x4 rr = u32x4{0u, 0u, 0u, 0u};
                        if (a.ep_res) rr = *(const u32x4*)(a.ep_res + e);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float lo = fmaf(__uint_as_float(v[q] << 16), mu[2 * q], rs[2 * q]) + __uint_as_float(rr[q] << 16);
                            float hi2 = fmaf(__uint_as_float(v[q] & 0xffff0000u), mu[2 * q + 1], rs[2 * q + 1]) + __uint_as_float(rr[q] & 0xffff0000u);
                            if (a.ep_relu) {
                                lo = lo > 0.f ? lo : 0.f;
                                hi2 = hi2 > 0.f ? hi2 : 0.f;
                            }
                            v[q] = pack_bf16x2(lo, hi2);
                        }
                    }
                } else if (fuse_mask) {   // ReLU mask of the layer below and its BatchNorm-backward sums, on the values as stored
                    const u32x4 ac = *(const u32x4*)(a.act + e);
                    u32x4 yy = u32x4{0u, 0u, 0u, 0u};
                    if (fuse_bn) yy = *(const u32x4*)(a.ybn + e);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float alo = __uint_as_float(ac[q] << 16), ahi = __uint_as_float(ac[q] & 0xffff0000u);
                        const float dlo = alo > 0.f ? __uint_as_float(v[q] << 16) : 0.f;
                        const float dhi = ahi > 0.f ? __uint_as_float(v[q] & 0xffff0000u) : 0.f;
                        v[q] = (alo > 0.f ? v[q] & 0xffffu : 0u) | (ahi > 0.f ? v[q] & 0xffff0000u : 0u);
                        f1[2 * q] += dlo;
                        f1[2 * q + 1] += dhi;
                        f2[2 * q] = fmaf(dlo, (__uint_as_float(yy[q] << 16) - mu[2 * q]) * rs[2 * q], f2[2 * q]);
                        f2[2 * q + 1] = fmaf(dhi, (__uint_as_float(yy[q] & 0xffff0000u) - mu[2 * q + 1]) * rs[2 * q + 1], f2[2 * q + 1]);
                    }
                }
                u32x4* dq = (u32x4*)(a.dst + e);
                if (STREAM) __builtin_nontemporal_store(v, dq);
                else *dq = v;
            }
        }
        tile = ntile;
    }

    if (do_stats || fuse_bn) {
        // lanes CV apart hold the same columns: fold them, then one slot per wavefront, fixed order over the slots
#pragma unroll
        for (int q = 0; q < FV; ++q) {
#pragma unroll
            for (int off = CV; off < 64; off <<= 1) {
                f1[q] += __shfl_xor(f1[q], off);
                f2[q] += __shfl_xor(f2[q], off);
            }
        }
        __syncthreads();
        if (lane < CV) {
#pragma unroll
            for (int q = 0; q < FV; ++q) {
                s_part[wave * BN + lane * 8 + q] = f1[q];
                s_part[(8 + wave) * BN + lane * 8 + q] = f2[q];
            }
        }
        __syncthreads();
        if (tid < 2 * BN) {
            const int stat = tid / BN, col = tid % BN;
            float v = 0.f;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) v += s_part[(stat * 8 + sl) * BN + col];
            prow[stat * BN + col] += v;   // (this block's row: zeroed above by the same thread)
        }
    }
}

// ---------------------------------------------------------------------------------
// The stem in its space-to-depth form (4 tap rows x 64 "channels" = 4 consecutive 16-value pixels, 64 output
// channels, forward only): K = 256 is four steps, so in the general kernel a tile is all prologue and epilogue.
// Same scheme as conv3x3_c64_kernel: the weights (32 KB) stay in LDS for all tiles of a block, the tile's input --
// the pixel range from the first output pixel's window to the end of the last one's, read once -- sits in LDS as a
// patch of 16-value pixels, a tap row is a pixel offset into it (the image carries its own zero border: no
// masks), and the next tile's patch travels through registers meanwhile.  A patch pixel takes 48 bytes (32 + 16):
// the fragment reads of 16 consecutive pixels then fall 12 banks apart, without conflicts.
static constexpr int STEM_BM = 256;
static constexpr int STEM_PPIX = 48;                          // bytes per patch pixel
static constexpr int STEM_PMAX = 1280;                        // patch pixels (the host checks the geometry against it)
static constexpr int STEM_NPP = (STEM_PMAX * 2 + 511) / 512;  // 16-byte patch pieces per thread
static constexpr int STEM_W_BYTES = 4 * 64 * 128;
static constexpr int STEM_PATCH_BYTES = STEM_PMAX * STEM_PPIX;
static constexpr int STEM_SMEM = STEM_W_BYTES + STEM_PATCH_BYTES + C64_CST_BYTES + C64_PART_BYTES;
static_assert(STEM_SMEM <= 160 * 1024, "LDS budget");

template <bool STREAM>
__global__ void __launch_bounds__(512) stem_s2d_kernel(IgemmArgs a) {
    constexpr int NT = 512, BM = STEM_BM, BN = 64, MI = 2, HM = 128, LDC = C64_LDC, PPIX = STEM_PPIX, NPP = STEM_NPP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;                                    // [4][64][8 positions of 16 bytes], swizzled
    unsigned char* s_patch = smem + STEM_W_BYTES;                 // [patch pixels][48 bytes]
    bf16_t* Cst = (bf16_t*)(s_patch + STEM_PATCH_BYTES);
    float* s_part = (float*)((unsigned char*)Cst + C64_CST_BYTES);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, hi = lane >> 5;
    const int Ws = a.Ws, Wd = a.Wd, hw_d = a.Hd * a.Wd, hw_s = a.Hs * a.Ws;
    const unsigned M = (unsigned)a.F * (unsigned)hw_d;            // output pixels
    const unsigned Min = (unsigned)a.F * (unsigned)hw_s;          // input pixels
    const int mtiles = (int)((M + BM - 1) / BM);
    const bool do_stats = a.stats != nullptr;
    const bool affine = a.ep_scale != nullptr;

    float* prow = do_stats ? a.stats + (size_t)blockIdx.x * 2 * BN : nullptr;
    if (prow && tid < 2 * BN) prow[tid] = 0.f;

    {
        const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(a.wp, (uint32_t)(BN * 256 * 2));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int q = tid + s * NT;                           // piece: tap row s, channel row n, position pos
            const int n = (q >> 3) & 63, pos = q & 7, kv = pos ^ ((n >> 1) & 7);
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, n * 512 + s * 128 + kv * 16, 0, 0);
            *(u32x4*)(s_w + q * 16) = v;
        }
    }

    // input pixel (frame f, row h, column w of the input image) under output pixel P = (f, h, w)
    auto pin_of = [&](unsigned P) {
        const unsigned f = P / (unsigned)hw_d, q = P - f * (unsigned)hw_d;
        const unsigned h = q / (unsigned)Wd, w = q - h * (unsigned)Wd;
        return f * (unsigned)hw_s + h * (unsigned)Ws + w;
    };
    // the patch of a tile: input pixels [pin_of(first), pin_of(last) + 3 rows + 4), two 16-byte pieces per pixel
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(a.src, (uint32_t)((long)Min * 32));
    u32x4 preg[NPP];
    auto load_patch = [&](int tile) {
        const unsigned P0 = (unsigned)tile * BM;
        const unsigned Pl = P0 + BM - 1 < M ? P0 + BM - 1 : M - 1;
        const unsigned pin0 = pin_of(P0);
        const int npx = (int)(pin_of(Pl) - pin0) + 3 * Ws + 4;
#pragma unroll
        for (int s = 0; s < NPP; ++s) {
            const int q = tid + s * NT;
            const bool ok = (q >> 1) < npx;   // (pixels behind the end of the tensor read as zeros)
            preg[s] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, ok ? (int)((pin0 + (unsigned)(q >> 1)) * 32u + (unsigned)(q & 1) * 16u) : (int)OOB_OFFSET, 0, 0);
        }
    };
    auto store_patch = [&]() {
#pragma unroll
        for (int s = 0; s < NPP; ++s) {
            const int q = tid + s * NT;
            *(u32x4*)(s_patch + (q >> 1) * PPIX + (q & 1) * 16) = preg[s];
        }
    };

    int b_rd[4];
    {
        const int n = wn * 32 + r;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) b_rd[ks] = n * 128 + (((2 * ks + hi) ^ ((n >> 1) & 7)) * 16);
    }

    constexpr int FV = 8, CV = BN / 8, RPS = NT / CV, NPS = HM / RPS;
    float f1[FV], f2[FV];
#pragma unroll
    for (int q = 0; q < FV; ++q) f1[q] = f2[q] = 0.f;
    const int vcol = tid % CV, r0 = tid / CV;
    float mu[FV], rs[FV];
#pragma unroll
    for (int q = 0; q < FV; ++q) mu[q] = rs[q] = 0.f;
    if (affine) {
#pragma unroll
        for (int q = 0; q < FV; ++q) {
            mu[q] = a.ep_scale[vcol * 8 + q];
            rs[q] = a.ep_shift[vcol * 8 + q];
        }
    }

    // an XCD takes a contiguous eighth of the tiles (see conv3x3_c64_kernel)
    const bool by_xcd = (gridDim.x % 8) == 0;
    const int per_xcd = by_xcd ? (mtiles + 7) / 8 : mtiles;
    const int xcd = by_xcd ? (int)(blockIdx.x % 8) : 0;
    const int seq_step = by_xcd ? (int)(gridDim.x / 8) : (int)gridDim.x;
    auto tile_at = [&](int seq) {
        const int t = xcd * per_xcd + seq;
        return (seq < per_xcd && t < mtiles) ? t : -1;
    };
    int seq = by_xcd ? (int)(blockIdx.x / 8) : (int)blockIdx.x;
    int tile = tile_at(seq);
    if (tile >= 0) load_patch(tile);
    __syncthreads();                      // weights, statistics row
    if (tile >= 0) store_patch();

    while (tile >= 0) {
        seq += seq_step;
        const int ntile = tile_at(seq);
        __syncthreads();                  // this tile's patch is in LDS

        // this lane's pixels: offset of their window's first pixel in the patch (rows beyond M compute on pixel 0)
        int a_base[MI];
        {
            const unsigned P0 = (unsigned)tile * BM;
            const unsigned pin0 = pin_of(P0);
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const unsigned P = P0 + (unsigned)(i * HM + wm * 32 + r);
                a_base[i] = (P < M ? (int)(pin_of(P) - pin0) : 0) * PPIX + hi * 16;
            }
        }

        f32x16 acc[MI];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

        if (ntile >= 0) load_patch(ntile);   // lands in registers while this tile is multiplied

#pragma unroll
        for (int tap = 0; tap < 4; ++tap) {
            const int toff = tap * Ws * PPIX;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {      // 16 of the tap row's 64 values: one pixel; lanes >= 32 take its second half
                const bf16x8 bfr = *(const bf16x8*)(s_w + tap * (64 * 128) + b_rd[ks]);
                bf16x8 af[MI];
#pragma unroll
                for (int i = 0; i < MI; ++i) af[i] = *(const bf16x8*)(s_patch + a_base[i] + toff + ks * PPIX);
#pragma unroll
                for (int i = 0; i < MI; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af[i], acc[i], 0, 0, 0);
            }
        }

        __syncthreads();                  // every wavefront has read its last fragment of the patch
        if (ntile >= 0) store_patch();

#pragma unroll
        for (int h = 0; h < MI; ++h) {
            if (h > 0) __syncthreads();
            {
                bf16_t* dstp = Cst + (wm * 32 + r) * LDC + wn * 32 + 4 * hi;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 w2;
                    w2.x = pack_bf16x2(acc[h][4 * q], acc[h][4 * q + 1]);
                    w2.y = pack_bf16x2(acc[h][4 * q + 2], acc[h][4 * q + 3]);
                    *(uint2*)(dstp + 8 * q) = w2;
                }
            }
            __syncthreads();
#pragma unroll
            for (int pss = 0; pss < NPS; ++pss) {
                const int row = pss * RPS + r0;
                const unsigned P = (unsigned)tile * BM + (unsigned)(h * HM + row);
                if (P >= M) continue;
                u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
                const long e = (long)P * BN + vcol * 8;
                if (do_stats) {   // statistics of the values as stored
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float lo = __uint_as_float(v[q] << 16), hi2 = __uint_as_float(v[q] & 0xffff0000u);
                        f1[2 * q] += lo;
                        f1[2 * q + 1] += hi2;
                        f2[2 * q] = fmaf(lo, lo, f2[2 * q]);
                        f2[2 * q + 1] = fmaf(hi2, hi2, f2[2 * q + 1]);
                    }
                }
                if (affine) {
                    u32x4 rr = u32x4{0u, 0u, 0u, 0u};
                    if (a.ep_res) rr = *(const u32x4*)(a.ep_res + e);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float lo = fmaf(__uint_as_float(v[q] << 16), mu[2 * q], rs[2 * q]) + __uint_as_float(rr[q] << 16);
                        float hi2 = fmaf(__uint_as_float(v[q] & 0xffff0000u), mu[2 * q + 1], rs[2 * q + 1]) + __uint_as_float(rr[q] & 0xffff0000u);
                        if (a.ep_relu) {
                            lo = lo > 0.f ? lo : 0.f;
                            hi2 = hi2 > 0.f ? hi2 : 0.f;
                        }
                        v[q] = pack_bf16x2(lo, hi2);
                    }
                }
                u32x4* dq = (u32x4*)(a.dst + e);
                if (STREAM) __builtin_nontemporal_store(v, dq);
                else *dq = v;
            }
        }
        tile = ntile;
    }

    if (do_stats) {
#pragma unroll
        for (int q = 0; q < FV; ++q) {
#pragma unroll
            for (int off = CV; off < 64; off <<= 1) {
                f1[q] += __shfl_xor(f1[q], off);
                f2[q] += __shfl_xor(f2[q], off);
            }
        }
        __syncthreads();
        if (lane < CV) {
#pragma unroll
            for (int q = 0; q < FV; ++q) {
                s_part[wave * BN + lane * 8 + q] = f1[q];
                s_part[(8 + wave) * BN + lane * 8 + q] = f2[q];
            }
        }
        __syncthreads();
        if (tid < 2 * BN) {
            const int stat = tid / BN, col = tid % BN;
            float v = 0.f;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) v += s_part[(stat * 8 + sl) * BN + col];
            prow[stat * BN + col] += v;
        }
    }
}

// ---------------------------------------------------------------------------------
// Two layers in one kernel, forward only, BatchNorm as a known per-channel affine map (inference): the 3x3
// convolution of a bottleneck (MID -> MID channels, any stride) and the 1x1 convolution behind it (MID -> 4*MID),
// for MID = 64 or 128.  The MID-channel tensor between them never leaves the chip:
//
//   phase 1  a 256-pixel tile of the 3x3 convolution, all MID output channels, as in igemm_ring_kernel: buffer-load
//            gathers, two LDS stages of A rows [256][64] and B rows [MID][64] in the same swizzled layout, the
//            next K step in flight in registers;
//   between  the accumulators go through the affine map and the ReLU (the convolution result rounded to bf16
//            first, the activation rounded once: what the two-kernel path stores) into the A parts of the stages,
//            64 channels per stage, in the fragment layout: they are now the A operand of
//   phase 2  the 1x1 convolution, 128 of its output channels at a time; only its weights move through the stages.
//            Every column tile ends with the affine map, the shortcut and the ReLU of the block's output and
//            16-byte stores, staged through LDS as in the other kernels.
//
// One block of eight wavefronts per CU; an XCD takes a contiguous eighth of the tiles (neighbouring tiles share the
// rows above and below a tile's pixels).
struct TailArgs {
    const bf16_t* src;        // [F][Hs][Ws][MID]: the activation in front of the 3x3 convolution
    const bf16_t* w2;         // packed [MID][9][MID]
    const bf16_t* w3;         // packed [4*MID][MID]
    const float *sc2, *sh2;   // [MID]: affine map behind the 3x3 convolution (ReLU follows)
    const float *sc3, *sh3;   // [4*MID]: affine map behind the 1x1 convolution
    const bf16_t* res;        // [F*Hd*Wd][4*MID]: added before the last ReLU
    bf16_t* dst;              // [F*Hd*Wd][4*MID]
    int F, Hs, Ws, Hd, Wd, stride;
};

template <int MID, bool STREAM>
__global__ void __launch_bounds__(512) fused_tail_kernel(TailArgs a) {
    constexpr int NT = 512, BM = 256, WN = 2, MI = 2, HM = 128;
    constexpr int BN1 = MID, TN1 = BN1 / WN, NJ1 = TN1 / 32;        // phase 1: all MID columns
    constexpr int BN2 = 128, TN2 = BN2 / WN, NJ2 = TN2 / 32;        // phase 2: 128 columns at a time
    constexpr int N2 = 4 * MID, NT2 = N2 / BN2, NK2 = MID / BK, CB = MID / BK;
    constexpr int ROWB = BK * 2;                                    // bytes per LDS row
    constexpr int STAGE = (BM + BN2) * ROWB;                        // A rows, then up to 128 B rows
    constexpr int LDC = BN2 + 8;
    constexpr int PA = BM / (NT / 8), PB1 = BN1 / (NT / 8), PB2 = BN2 / (NT / 8);
    constexpr int KS = BK / 16;
    static_assert(MID == 64 || MID == 128, "two stages hold the intermediate tile");
    static_assert(PA == 4 && PB2 == 2 && PB1 >= 1, "piece counts");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t* Cst = (bf16_t*)(smem + 2 * STAGE);                      // [HM][LDC]
    RowInfo* s_row = (RowInfo*)(Cst + HM * LDC);                    // [BM]
    float* s_aff = (float*)(s_row + BM);                            // sc2, sh2 [MID]; sc3, sh3 [N2]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = tid / 8;
    const int kvec = (tid % 8) ^ ((lrow >> 1) & 7);
    const int r = lane & 31, hi = lane >> 5;

    for (int c = tid; c < MID; c += NT) {
        s_aff[c] = a.sc2[c];
        s_aff[MID + c] = a.sh2[c];
    }
    for (int c = tid; c < N2; c += NT) {
        s_aff[2 * MID + c] = a.sc3[c];
        s_aff[2 * MID + N2 + c] = a.sh3[c];
    }

    const int hw_d = a.Hd * a.Wd, hw_s = a.Hs * a.Ws;
    const unsigned M = (unsigned)a.F * (unsigned)hw_d;
    const int mtiles = (int)((M + BM - 1) / BM);
    const int bias_el = (a.Ws + 1) * MID;                           // the most negative tap origin (pad 1)
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(a.src - bias_el, (uint32_t)(((long)a.F * hw_s * MID + bias_el) * 2));
    const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(a.w2, (uint32_t)(MID * 9 * MID * 2));
    const __amdgpu_buffer_rsrc_t rsrc_c = make_rsrc(a.w3, (uint32_t)(N2 * MID * 2));

    // fragment addresses inside a stage (see igemm_ring_kernel)
    int a_rd[KS], b_rd[KS];
    {
        const int sw = (r >> 1) & 7;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int pos = ((2 * ks + hi) ^ sw) * 16;
            a_rd[ks] = (wm * 32 + r) * ROWB + pos;
            b_rd[ks] = (BM + r) * ROWB + pos;                       // + (wn * TN + j * 32) rows
        }
    }

    // an XCD takes a contiguous eighth of the tiles
    const bool by_xcd = (gridDim.x % 8) == 0;
    const int per_xcd = by_xcd ? (mtiles + 7) / 8 : mtiles;
    const int xcd = by_xcd ? (int)(blockIdx.x % 8) : 0;
    const int seq_step = by_xcd ? (int)(gridDim.x / 8) : (int)gridDim.x;
    auto tile_at = [&](int seq) {
        const int t = xcd * per_xcd + seq;
        return (seq < per_xcd && t < mtiles) ? t : -1;
    };

    u32x4 greg[PA + PB2];
    uint32_t aoff[PA], amask[PA];

    // phase 1, K step k = (tap, 64-channel block): gathers of the A rows and the weights of the tap
    auto load1 = [&](int k) {
        const int tap = k / CB, chb = (k - tap * CB) * BK;
        const int th = tap / 3, tw = tap - th * 3;
        const uint32_t need = (1u << th) | (1u << (8 + tw));
        const int soff_a = ((th * a.Ws + tw) * MID + chb) * 2;
        const int soff_b = (tap * MID + chb) * 2;
#pragma unroll
        for (int i = 0; i < PA; ++i)
            greg[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, (int)((amask[i] & need) == need ? aoff[i] : OOB_OFFSET), soff_a, 0);
#pragma unroll
        for (int j = 0; j < PB1; ++j)
            greg[PA + j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, (int)((uint32_t)(j * (NT / 8) + lrow) * (9 * MID * 2) + kvec * 16), soff_b, 0);
    };
    auto store1 = [&](int stage) {
#pragma unroll
        for (int i = 0; i < PA; ++i) *(u32x4*)(smem + stage * STAGE + i * (NT / 8) * ROWB + tid * 16) = greg[i];
#pragma unroll
        for (int j = 0; j < PB1; ++j) *(u32x4*)(smem + stage * STAGE + (BM + j * (NT / 8)) * ROWB + tid * 16) = greg[PA + j];
    };
    // phase 2, step s = (column tile, 64-channel block): weights of the 1x1 convolution only
    auto load2 = [&](int s2) {
        const int nt = s2 / NK2, kk = s2 - nt * NK2;
#pragma unroll
        for (int j = 0; j < PB2; ++j)
            greg[PA + j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_c, (int)((uint32_t)(nt * BN2 + j * (NT / 8) + lrow) * (MID * 2) + kvec * 16), kk * BK * 2, 0);
    };
    auto store2 = [&](int stage) {
#pragma unroll
        for (int j = 0; j < PB2; ++j) *(u32x4*)(smem + stage * STAGE + (BM + j * (NT / 8)) * ROWB + tid * 16) = greg[PA + j];
    };

    __syncthreads();   // the affine vectors

    for (int seq = by_xcd ? (int)(blockIdx.x / 8) : (int)blockIdx.x, tile = tile_at(seq); tile >= 0; seq += seq_step, tile = tile_at(seq)) {
        // ---- rows of the tile: gather origin, tap validity, destination row
        if (tid < BM) {
            const unsigned m = (unsigned)tile * BM + tid;
            RowInfo info;
            info.off = 0;
            info.mask = 0;
            info.dst = -1;
            if (m < M) {
                const int f = (int)(m / (unsigned)hw_d);
                const int q = (int)(m - (unsigned)f * (unsigned)hw_d);
                const int dh = q / a.Wd, dw = q - dh * a.Wd;
                const int oh = dh * a.stride - 1, ow = dw * a.stride - 1;
                uint32_t mask = 0;
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    if (oh + t >= 0 && oh + t < a.Hs) mask |= 1u << t;
                    if (ow + t >= 0 && ow + t < a.Ws) mask |= 1u << (8 + t);
                }
                info.off = ((long)f * hw_s + (long)oh * a.Ws + ow) * MID;
                info.mask = mask;
                info.dst = (int)m;
            }
            s_row[tid] = info;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const RowInfo ri = s_row[i * (NT / 8) + lrow];
            aoff[i] = (uint32_t)((ri.off + bias_el) * 2) + kvec * 16;
            amask[i] = ri.mask;
        }

        // ---- phase 1
        f32x16 acc1[MI][NJ1];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ1; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc1[i][j][e] = 0.f;
        constexpr int NK1 = 9 * CB;
        load1(0);
        store1(0);
        __syncthreads();
        for (int k = 0; k < NK1; ++k) {
            const unsigned char* st = smem + (k & 1) * STAGE;
            if (k + 1 < NK1) load1(k + 1);
            else load2(0);                  // the first weights of phase 2 travel behind the last step
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 af[MI], bfr[NJ1];
#pragma unroll
                for (int i = 0; i < MI; ++i) af[i] = *(const bf16x8*)(st + a_rd[ks] + i * HM * ROWB);
#pragma unroll
                for (int j = 0; j < NJ1; ++j) bfr[j] = *(const bf16x8*)(st + b_rd[ks] + (wn * TN1 + j * 32) * ROWB);
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ1; ++j)
                        // operands swapped as in igemm_ring_kernel: the result block is [channel][pixel]
                        acc1[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc1[i][j], 0, 0, 0);
            }
            if (k + 1 < NK1) store1((k + 1) & 1);
            __syncthreads();
        }

        // ---- the intermediate tile: affine map + ReLU, into the A parts of the stages (64 channels per stage; with
        // 64 channels in all, stage 0).  Lane: pixel r of its row block, channels 8*q + 4*hi + {0..3} of its column block.
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int row = i * HM + wm * 32 + r;
            const int sw = (row >> 1) & 7;
#pragma unroll
            for (int j = 0; j < NJ1; ++j) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c0 = wn * TN1 + j * 32 + 8 * q + 4 * hi;      // first of four channels
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float y = bf16_to_f32(f32_to_bf16(acc1[i][j][4 * q + e]));
                        const float z = fmaf(y, s_aff[c0 + e], s_aff[MID + c0 + e]);
                        v[e] = z > 0.f ? z : 0.f;
                    }
                    uint2 w;
                    w.x = pack_bf16x2(v[0], v[1]);
                    w.y = pack_bf16x2(v[2], v[3]);
                    const int stage = c0 / BK, cv = (c0 % BK) / 8;
                    *(uint2*)(smem + stage * STAGE + row * ROWB + ((cv ^ sw) * 16) + (c0 & 4) * 2) = w;
                }
            }
        }
        store2(0);
        __syncthreads();

        // ---- phase 2
        constexpr int CV = BN2 / 8, RPS = NT / CV, NPS = HM / RPS;
        const int vcol = tid % CV, r0 = tid / CV;
        int s2 = 0;
        for (int nt = 0; nt < NT2; ++nt) {
            f32x16 acc2[MI][NJ2];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ2; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc2[i][j][e] = 0.f;
#pragma unroll
            for (int kk = 0; kk < NK2; ++kk, ++s2) {
                const bool more = s2 + 1 < NT2 * NK2;
                if (more) load2(s2 + 1);
                const unsigned char* sa = smem + (NK2 == 1 ? 0 : kk) * STAGE;    // the intermediate tile's 64-channel block
                const unsigned char* sb = smem + (s2 & 1) * STAGE;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    bf16x8 af[MI], bfr[NJ2];
#pragma unroll
                    for (int i = 0; i < MI; ++i) af[i] = *(const bf16x8*)(sa + a_rd[ks] + i * HM * ROWB);
#pragma unroll
                    for (int j = 0; j < NJ2; ++j) bfr[j] = *(const bf16x8*)(sb + b_rd[ks] + (wn * TN2 + j * 32) * ROWB);
#pragma unroll
                    for (int i = 0; i < MI; ++i)
#pragma unroll
                        for (int j = 0; j < NJ2; ++j)
                            acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc2[i][j], 0, 0, 0);
                }
                if (more) store2((s2 + 1) & 1);
                __syncthreads();
            }
            // epilogue of the column tile: scale / shift of this thread's eight columns, shortcut, ReLU
            const int col = nt * BN2 + vcol * 8;
            float sc[8], sh[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                sc[q] = s_aff[2 * MID + col + q];
                sh[q] = s_aff[2 * MID + N2 + col + q];
            }
#pragma unroll
            for (int h = 0; h < MI; ++h) {
                if (h > 0) __syncthreads();
                // the shortcut of this pass is requested before the staging
                u32x4 rr[NPS];
                int mrow[NPS];
#pragma unroll
                for (int pss = 0; pss < NPS; ++pss) {
                    mrow[pss] = s_row[h * HM + pss * RPS + r0].dst;
                    rr[pss] = *(const u32x4*)(mrow[pss] >= 0 ? a.res + (long)mrow[pss] * N2 + col : (const bf16_t*)g_zero_page);
                }
#pragma unroll
                for (int j = 0; j < NJ2; ++j) {
                    bf16_t* dstp = Cst + (wm * 32 + r) * LDC + wn * TN2 + j * 32 + 4 * hi;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint2 w;
                        w.x = pack_bf16x2(acc2[h][j][4 * q], acc2[h][j][4 * q + 1]);
                        w.y = pack_bf16x2(acc2[h][j][4 * q + 2], acc2[h][j][4 * q + 3]);
                        *(uint2*)(dstp + 8 * q) = w;
                    }
                }
                __syncthreads();
#pragma unroll
                for (int pss = 0; pss < NPS; ++pss) {
                    if (mrow[pss] < 0) continue;
                    u32x4 v = *(const u32x4*)(Cst + (pss * RPS + r0) * LDC + vcol * 8);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float lo = fmaf(__uint_as_float(v[e] << 16), sc[2 * e], sh[2 * e]) + __uint_as_float(rr[pss][e] << 16);
                        float hi2 = fmaf(__uint_as_float(v[e] & 0xffff0000u), sc[2 * e + 1], sh[2 * e + 1]) + __uint_as_float(rr[pss][e] & 0xffff0000u);
                        lo = lo > 0.f ? lo : 0.f;
                        hi2 = hi2 > 0.f ? hi2 : 0.f;
                        v[e] = pack_bf16x2(lo, hi2);
                    }
                    u32x4* dq = (u32x4*)(a.dst + (long)mrow[pss] * N2 + col);
                    if (STREAM) __builtin_nontemporal_store(v, dq);
                    else *dq = v;
                }
            }
        }
        __syncthreads();   // the row table and the stages are rewritten by the next tile
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
    if (p.stride > 2) return false;   // the dgrad kernel enumerates at most four parity classes
    if (p.KH > 8 || p.KW > 8) return false;        // tap-validity bit masks hold eight rows / columns
    if (p.KT > 1 && p.fold > 0) return false;      // frame offsets stay within one frame either way
    if (p.K() > 0x3fffffffL) return false;
    if (p.rows_in() * (long)p.Cin > 0x7fffffffL * 64 || p.rows_in() > 0x7fffffffL || p.rows_out() > 0x7fffffffL) return false;
    if ((long)p.H * p.W * p.Cin * (p.T + 2) > 0x7fffffffL || (long)p.Ho * p.Wo * p.Cout * (p.T + 2) > 0x7fffffffL) return false;
    return true;
}

// Fills the class table; returns the total number of M tiles.
static int setup_classes(IgemmArgs& a, bool dgrad, int BM) {
    if (!dgrad || a.stride == 1) {
        a.ncls = 1; a.cstep = 1;
        a.ph[0] = a.pw[0] = 0; a.hc[0] = a.Hd; a.wc[0] = a.Wd;
        a.a0h[0] = a.a0w[0] = 0; a.nth[0] = a.KH; a.ntw[0] = a.KW;
    } else {
        const int s = a.stride;
        a.ncls = s * s; a.cstep = s;
        for (int ph = 0; ph < s; ++ph)
            for (int pw = 0; pw < s; ++pw) {
                const int c = ph * s + pw;
                a.ph[c] = ph; a.pw[c] = pw;
                a.hc[c] = (a.Hd - ph + s - 1) / s;
                a.wc[c] = (a.Wd - pw + s - 1) / s;
                // destination row dh = ph (mod s) meets flipped tap a when (dh - padh + a) % s == 0
                a.a0h[c] = (((a.padh - ph) % s) + s) % s;
                a.a0w[c] = (((a.padw - pw) % s) + s) % s;
                a.nth[c] = a.a0h[c] < a.KH ? (a.KH - a.a0h[c] + s - 1) / s : 0;
                a.ntw[c] = a.a0w[c] < a.KW ? (a.KW - a.a0w[c] + s - 1) / s : 0;
                if (a.nth[c] == 0 || a.ntw[c] == 0) { a.nth[c] = a.ntw[c] = 0; }
            }
    }
    a.mt0[0] = 0;
    for (int c = 0; c < a.ncls; ++c) {
        const long Mc = (long)a.F * a.hc[c] * a.wc[c];
        a.mt0[c + 1] = a.mt0[c] + (int)((Mc + BM - 1) / BM);
    }
    for (int c = a.ncls; c < 4; ++c) {
        a.ph[c] = a.pw[c] = a.hc[c] = a.wc[c] = a.a0h[c] = a.a0w[c] = a.nth[c] = a.ntw[c] = 0;
        a.mt0[c + 1] = a.mt0[a.ncls];
    }
    return a.mt0[a.ncls];
}

// ---------------------------------------------------------------------------------
// 1x1, stride 1, KC = 64 or 128 -> 256 or 512 channels, forward with the statistics epilogue (the last convolution of
// the first two stages' blocks, the first stage's projection): four bytes written per byte read, one or two K steps.
// In the general kernel a tile of such a layer is all prologue, barriers and epilogue; here nothing is shared between
// wavefronts but the weights:
//
//  * the weights of 256 result channels (32 or 64 KB) sit in LDS for the life of the block, swizzled; a result of 512
//    channels is split over pairs of neighbouring blocks, which read the same rows of the input;
//  * a wavefront takes 32 pixels at a time: its A operand comes straight from memory in fragment order (lane = pixel
//    lane % 32, K vector 2*ks + lane / 32: the 32 rows of 128 or 256 bytes are one contiguous piece), the next pass's
//    fragments are requested before this pass is multiplied;
//  * 128 output channels at a time go through a staging tile that belongs to the wavefront alone (no block barrier
//    anywhere in the loop) and leave as 16-byte stores, 256 contiguous bytes per pixel row; the statistics are taken
//    from the staged values, eight fixed channels per lane, reduced once at the end of the block.
// Partial rows (a.stats, [gridDim.x][2][Cd]): row s of the first gridDim.x / nsplit rows receives the sums of stream s,
// the others are written as zeros (callers size and sum the rows by the general kernel's grid).
static constexpr int PW_LDC = 128 + 8;                        // staging pitch (elements)
static constexpr int PW_CST_BYTES = 32 * PW_LDC * 2;          // per wavefront
static constexpr int PW_PART_BYTES = 2 * 8 * 256 * 4;
static_assert(PW_CST_BYTES % 16 == 0, "alignment");
template <int KC>
struct PwD {
    static constexpr int ROWB = KC * 2;                        // bytes per weight row
    static constexpr int NB = KC <= 128 ? 256 : 128;           // result channels per block (64 KB of weights at most)
    static constexpr int NH = NB / 128;                        // passes of 128 result channels
    static constexpr int W_BYTES = NB * ROWB;
    static constexpr int SMEM = W_BYTES + 8 * PW_CST_BYTES + PW_PART_BYTES;
};
static_assert(PwD<128>::SMEM <= 160 * 1024 && PwD<256>::SMEM <= 160 * 1024, "LDS budget");

// Block index -> (stream of pixels, part of the result channels).  The nsplit blocks that share a stream read the same
// rows of the operand: they get indices 8 apart inside a run of 8 * nsplit, so that they share an XCD (workgroups go to
// the XCDs round-robin by index) and its L2.  Grids that are not a multiple of 8 * nsplit: neighbouring indices.
__device__ __forceinline__ void pw_block_role(int nsplit, int* stream, int* part) {
    const int bid = (int)blockIdx.x;
    if (nsplit > 1 && (int)gridDim.x % (8 * nsplit) == 0) {
        const int local = bid >> 3;
        *part = local % nsplit;
        *stream = (local / nsplit) * 8 + (bid & 7);
    } else {
        *part = bid % nsplit;
        *stream = bid / nsplit;
    }
}

// AFF: the affine epilogue of IgemmArgs::ep_scale (inference: BatchNorm with known statistics, optional residual and
// ReLU), applied to the staged values as igemm_ring_kernel applies it; the residual pieces of a pass are requested ahead
// of the staging of the accumulators.
template <int KC, bool STREAM, bool AFF = false>
__global__ void __launch_bounds__(512) pw_fwd_kernel(IgemmArgs a) {
    constexpr int LDC = PW_LDC, KS = KC / 16, ROWB = PwD<KC>::ROWB, KV = KC / 8, NB = PwD<KC>::NB, NH = PwD<KC>::NH;
    constexpr bool DB = KC <= 128;                                 // the next pass's fragments in registers of their own
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;                                                       // [NB][KV positions of 16 bytes]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bf16_t* Cst = (bf16_t*)(smem + PwD<KC>::W_BYTES + wave * PW_CST_BYTES);          // [32][LDC], this wavefront's
    float* s_part = (float*)(smem + PwD<KC>::W_BYTES + 8 * PW_CST_BYTES);            // [2 stats][8 wavefronts][NB]
    const int r = lane & 31, hi = lane >> 5;
    const long M = (long)a.F * a.Hd * a.Wd;
    const bool do_stats = a.stats != nullptr;
    const int nsplit = a.Cd / NB;
    int row_s, part;
    pw_block_role(nsplit, &row_s, &part);
    const int nb0 = part * NB;                                     // first result channel of this block
    const long stream0 = (long)row_s * 8 + wave;
    const long nstreams = (long)((int)gridDim.x / nsplit) * 8;
    // position p of weight row n holds K vector p ^ swz(n): the 16 (or 2 x 8) rows that one quarter-wave reads together
    // then lie in 16 different 16-byte bank groups
    auto swz = [](int n) { return KC >= 128 ? (n & 15) : ((n >> 1) & 7); };

    {
        const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(a.wp + (long)nb0 * KC, (uint32_t)(NB * ROWB));
#pragma unroll
        for (int q4 = 0; q4 < NB * KV / 512; ++q4) {
            const int q = tid + q4 * 512;                          // piece: weight row n, position pos
            const int n = q / KV, pos = q % KV, kv = pos ^ swz(n);
            *(u32x4*)(s_w + q * 16) = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, n * ROWB + kv * 16, 0, 0);
        }
    }
    __syncthreads();

    int b_rd[KS];                                                  // fragment of weight rows 32*j + r, step ks
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) b_rd[ks] = r * ROWB + (((2 * ks + hi) ^ swz(r)) << 4);
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(a.src, (uint32_t)(M * ROWB));
    const long nslabs = (M + 31) / 32;
    auto load_a = [&](long sl, bf16x8* fr) {
        const long row = sl * 32 + r;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, row < M ? (int)(row * ROWB + (2 * ks + hi) * 16) : (int)OOB_OFFSET, 0, 0);
            fr[ks] = __builtin_bit_cast(bf16x8, v);
        }
    };
    float f1[NH][8], f2[NH][8];
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int q = 0; q < 8; ++q) f1[h][q] = f2[h][q] = 0.f;
    const int vcol = lane & 15, row0 = lane >> 4;                  // store loop: piece lane + 64*t is row row0 + 4*t, vector vcol
    float sc[AFF ? NH : 1][8], sh[AFF ? NH : 1][8];                // AFF: scale and shift of this lane's channels
    if (AFF) {
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                sc[AFF ? h : 0][q] = a.ep_scale[nb0 + h * 128 + vcol * 8 + q];
                sh[AFF ? h : 0][q] = a.ep_shift[nb0 + h * 128 + vcol * 8 + q];
            }
    }
    const bf16_t* zero_page_f = (const bf16_t*)g_zero_page;

    long slab = stream0;
    bf16x8 cur[KS], nxt[DB ? KS : 1];
    if (slab < nslabs) load_a(slab, cur);
    for (; slab < nslabs; slab += nstreams) {
        if (DB && slab + nstreams < nslabs) load_a(slab + nstreams, nxt);
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            f32x16 acc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bf16x8 bfrag = *(const bf16x8*)(s_w + (h * 4 + j) * 32 * ROWB + b_rd[ks]);
                    // operands swapped as in igemm_ring_kernel: the result block is [channel][pixel]
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, cur[ks], acc[j], 0, 0, 0);
                }
            // (long K: the next pass's fragments take the place of this pass's, which the last product has read)
            if (!DB && h == NH - 1 && slab + nstreams < nslabs) load_a(slab + nstreams, cur);
            constexpr int RG = KC == 256 ? 8 : 4;                  // AFF: residual pieces requested together (registers)
            u32x4 rr[AFF ? RG : 1];
            auto request = [&](int g) {
#pragma unroll
                for (int t = 0; t < RG; ++t) {
                    const long grow = slab * 32 + row0 + 4 * (g * RG + t);
                    // (a load without a branch around it: rows that are not stored read the zero page)
                    rr[AFF ? t : 0] = *(const u32x4*)((a.ep_res && grow < M) ? a.ep_res + grow * a.Cd + nb0 + h * 128 + vcol * 8 : zero_page_f);
                }
            };
            if (AFF) request(0);
            // lane: pixel r, channels 32*j + 8*q + 4*hi + {0..3}
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16_t* dstp = Cst + r * LDC + j * 32 + 4 * hi;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint2 w;
                    w.x = pack_bf16x2(acc[j][4 * q], acc[j][4 * q + 1]);
                    w.y = pack_bf16x2(acc[j][4 * q + 2], acc[j][4 * q + 3]);
                    *(uint2*)(dstp + 8 * q) = w;
                }
            }
            __builtin_amdgcn_wave_barrier();                       // (LDS serves a wavefront's accesses in order)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int row = row0 + 4 * t;
                const long grow = slab * 32 + row;
                u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
                if (grow < M) {
                    if (do_stats) {   // statistics of the values as stored
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float lo = __uint_as_float(v[e] << 16), hv = __uint_as_float(v[e] & 0xffff0000u);
                            f1[h][2 * e] += lo;
                            f1[h][2 * e + 1] += hv;
                            f2[h][2 * e] = fmaf(lo, lo, f2[h][2 * e]);
                            f2[h][2 * e + 1] = fmaf(hv, hv, f2[h][2 * e + 1]);
                        }
                    }
                    if (AFF) {
                        const u32x4 rv = rr[AFF ? t % RG : 0];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float lo = fmaf(__uint_as_float(v[e] << 16), sc[AFF ? h : 0][2 * e], sh[AFF ? h : 0][2 * e]) + __uint_as_float(rv[e] << 16);
                            float hv = fmaf(__uint_as_float(v[e] & 0xffff0000u), sc[AFF ? h : 0][2 * e + 1], sh[AFF ? h : 0][2 * e + 1]) + __uint_as_float(rv[e] & 0xffff0000u);
                            if (a.ep_relu) {
                                lo = lo > 0.f ? lo : 0.f;
                                hv = hv > 0.f ? hv : 0.f;
                            }
                            v[e] = pack_bf16x2(lo, hv);
                        }
                    }
                    u32x4* q = (u32x4*)(a.dst + grow * a.Cd + nb0 + h * 128 + vcol * 8);
                    if (STREAM) __builtin_nontemporal_store(v, q);
                    else *q = v;
                }
                if (AFF && RG < 8 && t == RG - 1) request(1);
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (DB) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) cur[ks] = nxt[DB ? ks : 0];
        }
    }
    if (do_stats) {
        // lanes 16 apart hold the same columns: fold them, then one slot per wavefront, fixed order over the slots
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                f1[h][q] += __shfl_xor(f1[h][q], 16);
                f2[h][q] += __shfl_xor(f2[h][q], 16);
                f1[h][q] += __shfl_xor(f1[h][q], 32);
                f2[h][q] += __shfl_xor(f2[h][q], 32);
            }
        if (lane < 16) {
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    s_part[wave * NB + h * 128 + lane * 8 + q] = f1[h][q];
                    s_part[(8 + wave) * NB + h * 128 + lane * 8 + q] = f2[h][q];
                }
        }
        __syncthreads();
        if (tid < 2 * NB) {
            const int stat = tid / NB, c = tid % NB;
            float v = 0.f;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) v += s_part[(stat * 8 + sl) * NB + c];
            const int rows_used = (int)gridDim.x / nsplit;
            a.stats[((size_t)row_s * 2 + stat) * a.Cd + nb0 + c] = v;
            for (int rz = rows_used + row_s; rz < (int)gridDim.x; rz += rows_used)      // rows beyond the streams: zeros
                a.stats[((size_t)rz * 2 + stat) * a.Cd + nb0 + c] = 0.f;
        }
    }
}

// ---------------------------------------------------------------------------------
// The same scheme for the data gradient of a block's first convolution where it is short in K and wide in its result
// (1x1, stride 1, KC = 64 or 128 channels of dy -> 256 or 512 channels of dx): these tiles carry, besides the
// convolution, three tensors of the result's size through the epilogue -- the shortcut gradient, the BatchNorm input of
// the block below and the result itself -- so the layer is a stream with a small product attached.  A block holds the
// weights of 256 result channels (a result of 512 channels is split over pairs of neighbouring blocks, which read the
// same rows of dy); a wavefront takes 32 pixels at a time, 128 result channels at a time through its own staging tile.
// The stored values are those of igemm_ring_kernel's data gradient, value for value: adjoint shift as a frame offset on
// the destination row (a lane's eight channels lie in one shift group), zero value for the frame a group leaves empty,
// shortcut gradient added, mask from the decision bits.  The BatchNorm-backward sums of the stored values are taken in
// a different order (raw sums in the loop, mean and rstd applied once per block: see f1, f2 below).  The operands of
// four or eight destination pieces are requested together: the kernel is bound by the bytes a CU has in flight.
// Partial rows (a.stats, [gridDim.x][2][Cd]): row s of the first gridDim.x / nsplit rows receives the sums of stream s,
// the others are written as zeros (callers size and sum the rows by the general kernel's grid).
// CADD: the shortcut gradient comes in the compact form described at IgemmArgs::add_stride.
template <int KC, bool STREAM, bool CADD = false>
__global__ void __launch_bounds__(512) pw_dgrad_kernel(IgemmArgs a) {
    constexpr int LDC = PW_LDC, KS = KC / 16, ROWB = PwD<KC>::ROWB, KV = KC / 8, NB = PwD<KC>::NB, NH = PwD<KC>::NH;
    constexpr int GP = KC == 64 ? 8 : 4;                           // destination pieces requested together (registers)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;                                                       // [NB][KV positions of 16 bytes]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bf16_t* Cst = (bf16_t*)(smem + PwD<KC>::W_BYTES + wave * PW_CST_BYTES);          // [32][LDC], this wavefront's
    float* s_part = (float*)(smem + PwD<KC>::W_BYTES + 8 * PW_CST_BYTES);            // [2 sums][8 wavefronts][NB]
    const int r = lane & 31, hi = lane >> 5;
    const int hw = a.Hd * a.Wd;
    const long M = (long)a.F * hw;
    const int nsplit = a.Cd / NB;
    int row_s, part;
    pw_block_role(nsplit, &row_s, &part);
    const int nb0 = part * NB;                                     // first result channel of this block
    const long stream0 = (long)row_s * 8 + wave;
    const long nstreams = (long)((int)gridDim.x / nsplit) * 8;
    const bool fuse_mask = a.act_bits != nullptr;
    const bool fuse_bn = fuse_mask && a.ybn != nullptr;
    // position p of weight row n holds K vector p ^ swz(n): the 16 (or 2 x 8) rows that one quarter-wave reads together
    // then lie in 16 different 16-byte bank groups
    auto swz = [](int n) { return KC >= 128 ? (n & 15) : ((n >> 1) & 7); };

    {
        const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(a.wp + (long)nb0 * KC, (uint32_t)(NB * ROWB));
#pragma unroll
        for (int q4 = 0; q4 < NB * KV / 512; ++q4) {
            const int q = tid + q4 * 512;                          // piece: weight row n, position pos
            const int n = q / KV, pos = q % KV, kv = pos ^ swz(n);
            *(u32x4*)(s_w + q * 16) = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, n * ROWB + kv * 16, 0, 0);
        }
    }
    __syncthreads();

    int b_rd[KS];                                                  // fragment of weight rows 32*j + r, step ks
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) b_rd[ks] = r * ROWB + (((2 * ks + hi) ^ swz(r)) << 4);
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(a.src, (uint32_t)(M * ROWB));
    const long nslabs = (M + 31) / 32;
    bf16x8 cur[KS];
    auto load_a = [&](long sl) {
        const long row = sl * 32 + r;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, row < M ? (int)(row * ROWB + (2 * ks + hi) * 16) : (int)OOB_OFFSET, 0, 0);
            cur[ks] = __builtin_bit_cast(bf16x8, v);
        }
    };
    // store loop: piece lane + 64*t of a 32 x 128 half is row row0 + 4*t, vector vcol: a lane's channels never change
    const int vcol = lane & 15, row0 = lane >> 4;
    // BatchNorm-backward sums: f1 = sum(dz), f2 = sum(dz * y) with the raw BatchNorm input; the block turns the second
    // into sum(dz * (y - mean) * rstd) = (f2 - mean * f1) * rstd once, when it writes its partial row (the mean and rstd
    // of a lane's sixteen channels would cost the loop 32 registers, which it spends on operands in flight instead)
    float f1[NH][8], f2[NH][8];
    int dt[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        dt[h] = group_dt(nb0 + h * 128 + vcol * 8, a.fold);
#pragma unroll
        for (int q = 0; q < 8; ++q) f1[h][q] = f2[h][q] = 0.f;
    }
    const bf16_t* zero_page = (const bf16_t*)g_zero_page;

    long slab = stream0;
    if (slab < nslabs) load_a(slab);
    for (; slab < nslabs; slab += nstreams) {
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const int col = nb0 + h * 128 + vcol * 8;
            f32x16 acc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bf16x8 bfrag = *(const bf16x8*)(s_w + (h * 4 + j) * 32 * ROWB + b_rd[ks]);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, cur[ks], acc[j], 0, 0, 0);
                }
            // the next pass's fragments: this pass has no further use for the registers
            if (h == NH - 1 && slab + nstreams < nslabs) load_a(slab + nstreams);
            // value (+ addend) -> optional mask and BatchNorm sums -> store, as igemm_ring_kernel's data gradient
            auto finish = [&](int mr, u32x4 o, const u32x4& ad, uint32_t bits, const u32x4& yy) {
                if (a.addend) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float lo = __uint_as_float(o[q] << 16) + __uint_as_float(ad[q] << 16);
                        const float hv = __uint_as_float(o[q] & 0xffff0000u) + __uint_as_float(ad[q] & 0xffff0000u);
                        o[q] = pack_bf16x2(lo, hv);
                    }
                }
                if (fuse_mask) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const bool plo = ((bits >> (2 * q)) & 1u) != 0, phi = ((bits >> (2 * q + 1)) & 1u) != 0;
                        const float dlo = plo ? __uint_as_float(o[q] << 16) : 0.f;
                        const float dhi = phi ? __uint_as_float(o[q] & 0xffff0000u) : 0.f;
                        o[q] = (plo ? o[q] & 0xffffu : 0u) | (phi ? o[q] & 0xffff0000u : 0u);
                        f1[h][2 * q] += dlo;
                        f1[h][2 * q + 1] += dhi;
                        f2[h][2 * q] = fmaf(dlo, __uint_as_float(yy[q] << 16), f2[h][2 * q]);
                        f2[h][2 * q + 1] = fmaf(dhi, __uint_as_float(yy[q] & 0xffff0000u), f2[h][2 * q + 1]);
                    }
                }
                u32x4* qd = (u32x4*)(a.dst + (long)mr * a.Cd + col);
                if (STREAM) __builtin_nontemporal_store(o, qd);
                else *qd = o;
            };
            // lane: pixel r, channels 32*j + 8*q + 4*hi + {0..3}
            auto stage = [&]() {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bf16_t* dstp = Cst + r * LDC + j * 32 + 4 * hi;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint2 w;
                        w.x = pack_bf16x2(acc[j][4 * q], acc[j][4 * q + 1]);
                        w.y = pack_bf16x2(acc[j][4 * q + 2], acc[j][4 * q + 3]);
                        *(uint2*)(dstp + 8 * q) = w;
                    }
                }
                __builtin_amdgcn_wave_barrier();                   // (LDS serves a wavefront's accesses in order)
            };
            // the first group's operands are requested ahead of the staging of the accumulators; where all eight pieces
            // are requested at once the accumulators go first, to make room for them
            if (GP == 8) stage();
#pragma unroll
            for (int g = 0; g < 8 / GP; ++g) {                     // groups of GP pieces
                int mr[GP], mz[GP];
                int arow[CADD ? GP : 1];                           // the pixel's row in the compact addend, or -1
                u32x4 ad[GP], yy[GP];
                uint32_t bt[GP];
#pragma unroll
                for (int t = 0; t < GP; ++t) {
                    const long grow = slab * 32 + row0 + 4 * (GP * g + t);
                    const bool live = grow < M;
                    const unsigned fr = CADD && live ? (unsigned)grow / (unsigned)hw : 0u;
                    const int tt = CADD ? (int)(fr % (unsigned)a.T) : (live ? (int)((grow / hw) % a.T) : 0);
                    const bool in_clip = tt + dt[h] >= 0 && tt + dt[h] < a.T;
                    mr[t] = live && in_clip ? (int)grow + dt[h] * hw : -1;
                    mz[t] = live && ((dt[h] == 1 && tt == 0) || (dt[h] == -1 && tt == a.T - 1)) ? (int)grow : -1;
                    // loads without a branch around them (rows that are not stored read the zero page)
                    const long e = (long)mr[t] * a.Cd + col;
                    const bool ok = mr[t] >= 0;
                    if (CADD) {
                        // (the frame offset of the adjoint shift does not change the pixel)
                        const unsigned q = (unsigned)grow - fr * (unsigned)hw;
                        const unsigned ph = q / (unsigned)a.Wd, pw = q - ph * (unsigned)a.Wd;
                        arow[t] = live && ((ph | pw) & 1u) == 0 ? (int)((fr * (unsigned)a.add_ho + (ph >> 1)) * (unsigned)a.add_wo + (pw >> 1)) : -1;
                        const long ea = ((long)arow[t] + (long)dt[h] * (a.add_ho * a.add_wo)) * a.Cd + col;
                        ad[t] = *(const u32x4*)((ok && arow[t] >= 0) ? a.addend + ea : zero_page);
                    } else {
                        ad[t] = *(const u32x4*)((ok && a.addend) ? a.addend + e : zero_page);
                    }
                    bt[t] = *((ok && fuse_mask) ? a.act_bits + e / 8 : (const uint8_t*)zero_page);
                    yy[t] = *(const u32x4*)((ok && fuse_bn) ? a.ybn + e : zero_page);
                }
                if (GP < 8 && g == 0) stage();
#pragma unroll
                for (int t = 0; t < GP; ++t) {
                    const int row = row0 + 4 * (GP * g + t);
                    const u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
                    if (mr[t] >= 0) finish(mr[t], v, ad[t], bt[t], yy[t]);
                }
#pragma unroll
                for (int t = 0; t < GP; ++t) {                     // the frame that receives nothing from inside the clip
                    if (mz[t] < 0) continue;
                    const long e = (long)mz[t] * a.Cd + col;
                    u32x4 zad = u32x4{0u, 0u, 0u, 0u}, zyy = zad;
                    uint32_t zbt = 0;
                    if (CADD) {
                        if (arow[t] >= 0) zad = *(const u32x4*)(a.addend + (long)arow[t] * a.Cd + col);
                    } else if (a.addend) {
                        zad = *(const u32x4*)(a.addend + e);
                    }
                    if (fuse_mask) zbt = a.act_bits[e / 8];
                    if (fuse_bn) zyy = *(const u32x4*)(a.ybn + e);
                    finish(mz[t], u32x4{0u, 0u, 0u, 0u}, zad, zbt, zyy);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    if (a.stats) {
        // lanes 16 apart hold the same columns: fold them, then one slot per wavefront, fixed order over the slots
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                f1[h][q] += __shfl_xor(f1[h][q], 16);
                f2[h][q] += __shfl_xor(f2[h][q], 16);
                f1[h][q] += __shfl_xor(f1[h][q], 32);
                f2[h][q] += __shfl_xor(f2[h][q], 32);
            }
        if (lane < 16) {
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    s_part[wave * NB + h * 128 + lane * 8 + q] = f1[h][q];
                    s_part[(8 + wave) * NB + h * 128 + lane * 8 + q] = f2[h][q];
                }
        }
        __syncthreads();
        if (tid < 2 * NB) {
            const int stat = tid / NB, c = tid % NB;
            float v1 = 0.f, v2 = 0.f;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) {
                v1 += s_part[sl * NB + c];
                v2 += s_part[(8 + sl) * NB + c];
            }
            if (fuse_bn) v2 = (v2 - a.bn_mean[nb0 + c] * v1) * a.bn_rstd[nb0 + c];
            const int rows_used = (int)gridDim.x / nsplit;
            a.stats[((size_t)row_s * 2 + stat) * a.Cd + nb0 + c] = stat ? v2 : v1;
            // rows beyond the streams: zeros (each block clears its own channels in the rows congruent to its stream)
            for (int rz = rows_used + row_s; rz < (int)gridDim.x; rz += rows_used)
                a.stats[((size_t)rz * 2 + stat) * a.Cd + nb0 + c] = 0.f;
        }
    }
}

// Persistent grid: `per_cu` blocks per CU (a multiple of 8 blocks so that a block stays on one XCD), capped
// by the number of tile ids, which enumerate (group of 8 M tiles) x N tiles x (xcd).
static int igemm_grid(int mtiles, int Cd, int BN, int per_cu) {
    const int ntiles = (Cd + BN - 1) / BN;
    const int total = ((mtiles + 7) / 8) * 8 * ntiles;
    int grid = per_cu * num_cu();
    grid = (grid / 8) * 8;
    if (grid > total) grid = total;
    if (grid < 1) grid = 1;
    return grid;
}

template <int BM, int BN, int WM, int WN, bool DGRAD, int PF, int MINB>
static int launch_igemm(IgemmArgs& a, const char* name, hipStream_t s) {
    const int mtiles = setup_classes(a, DGRAD, BM);
    a.ntiles = (a.Cd + BN - 1) / BN;
    size_t smem = (size_t)2 * (BM + BN) * LDK * sizeof(bf16_t) + (size_t)2 * BM * sizeof(RowInfo);
    auto kern = igemm_kernel<BM, BN, WM, WN, DGRAD, PF, MINB>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "igemm: cannot raise dynamic LDS limit");
        configured = true;
    }
    const int grid = igemm_grid(mtiles, a.Cd, BN, MINB);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, s, a);
    return check_launch(name);   // class names carry the tile shape so that they map one-to-one onto kernel symbols
}

template <int BM, int BN, int WM, int WN, bool DGRAD, bool STREAM, bool CADD = false, bool MBITS = false>
static int launch_igemm_ring_s(IgemmArgs& a, const char* name, hipStream_t s) {
    const int mtiles = setup_classes(a, DGRAD, BM);
    a.ntiles = (a.Cd + BN - 1) / BN;
    // two operand stages, staging tile of one epilogue pass, statistics slots, two row buffers
    const size_t smem = (size_t)2 * (BM + BN) * BK * sizeof(bf16_t) + (BN == 256 ? 0 : (size_t)(WM * 32) * (BN + 8) * sizeof(bf16_t)) +
                        (size_t)2 * WM * WN * BN * sizeof(float) + (size_t)2 * BM * sizeof(RowInfo) + (size_t)2 * BM * sizeof(int);
    static_assert((size_t)2 * (BM + BN) * BK * sizeof(bf16_t) + (BN == 256 ? 0 : (size_t)(WM * 32) * (BN + 8) * sizeof(bf16_t)) +
                  (size_t)2 * WM * WN * BN * sizeof(float) + (size_t)2 * BM * sizeof(RowInfo) + (size_t)2 * BM * sizeof(int) <= 160 * 1024, "LDS budget");
    auto kern = igemm_ring_kernel<BM, BN, WM, WN, DGRAD, STREAM, CADD, MBITS>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "igemm: cannot raise dynamic LDS limit");
        configured = true;
    }
    const int grid = igemm_grid(mtiles, a.Cd, BN, 1);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), smem, s, a);
    return check_launch(name);
}

// Results far larger than the caches are stored past them (the next reader would not find them there anyway,
// and what is cached survives); smaller ones take the normal path.
template <int BM, int BN, int WM, int WN, bool DGRAD>
static int launch_igemm_ring(IgemmArgs& a, const char* name, hipStream_t s) {
    const bool stream = (long)a.F * a.Hd * a.Wd * a.Cd * 2 > (64L << 20);
    if constexpr (DGRAD && !(BM == 256 && BN == 64)) {
        // variants of the data gradient: compact addend, mask from decision bits (outputs of at most 64 channels carry
        // neither a projection's gradient nor a block output's mask)
        const bool cadd = a.add_stride == 2, mbits = a.act_bits != nullptr;
        if (!mbits) a.act_bits = nullptr;
        if (cadd && mbits)
            return stream ? launch_igemm_ring_s<BM, BN, WM, WN, true, true, true, true>(a, name, s)
                          : launch_igemm_ring_s<BM, BN, WM, WN, true, false, true, true>(a, name, s);
        if (cadd)
            return stream ? launch_igemm_ring_s<BM, BN, WM, WN, true, true, true, false>(a, name, s)
                          : launch_igemm_ring_s<BM, BN, WM, WN, true, false, true, false>(a, name, s);
        if (mbits)
            return stream ? launch_igemm_ring_s<BM, BN, WM, WN, true, true, false, true>(a, name, s)
                          : launch_igemm_ring_s<BM, BN, WM, WN, true, false, false, true>(a, name, s);
    } else {
        if (a.add_stride == 2) return fail(TSM_ERR_UNSUPPORTED, "igemm: no compact addend on this tile");
        a.act_bits = nullptr;   // this tile takes the mask from the activation
    }
    if (stream) return launch_igemm_ring_s<BM, BN, WM, WN, DGRAD, true>(a, name, s);
    return launch_igemm_ring_s<BM, BN, WM, WN, DGRAD, false>(a, name, s);
}

// Tile choice.  The ring kernel (one block of eight wavefronts per CU; 256x128 tiles, 256x64 for outputs of at
// most 64 channels) takes every layer whose source channels are a multiple of 64 and whose tensors stay below
// the 2 GiB that its 32-bit buffer offsets address; the rest goes to the register-prefetch kernels, two blocks
// per CU: 128x64 tiles for narrow outputs (<= 64 channels), 128x128 otherwise.
// `needed`: the layer has a pixel pitch other than its channel count (the stem in space-to-depth form), which only
// this kernel handles, so the comparison switch does not apply to it.
static bool ring_eligible(int Cs, long src_elems, long w_elems, bool needed) {
    static int enabled = -1;   // TSM_IGEMM_RING=0 keeps the register-prefetch kernels wherever they can run (for comparisons)
    if (enabled < 0) {
        const char* e = getenv("TSM_IGEMM_RING");
        enabled = (e && e[0] == '0') ? 0 : 1;
    }
    const long limit = 0x7ff00000L;   // bytes, leaves room for the padding bias in front of the tensor
    return (enabled || needed) && Cs % BK == 0 && src_elems * 2 < limit && w_elems * 2 < limit;
}

// Rows per tile of the ring kernel: 256, or 128 when 256-row tiles would leave a good part of the CUs without
// a tile (small batches in the last stages).
static int ring_rows(long rows, int Cd) {
    static int forced = -1;   // TSM_IGEMM_BM=128|256 fixes the choice (for comparisons)
    if (forced < 0) {
        const char* e = getenv("TSM_IGEMM_BM");
        forced = e ? atoi(e) : 0;
    }
    if (forced == 128 || forced == 256) return forced;
    const long ntiles = (Cd + 127) / 128;
    const long tiles256 = ((rows + 255) / 256) * (Cd <= 64 ? 1 : ntiles);
    return tiles256 * 4 < (long)num_cu() * 3 ? 128 : 256;
}

// Columns per tile of the ring kernel: 128, or 64 for outputs of at most 64 channels and where even 128-row tiles
// with 128 columns would leave a good part of the CUs without a tile (the last stage at the paper's batch of 8
// clips: 25 row tiles x 4 column tiles for 256 CUs).  TSM_IGEMM_NARROW=0 keeps 128 columns (for comparisons).
static int ring_cols(long rows, int Cd) {
    if (Cd <= 64) return 64;
    static int enabled = -1;
    if (enabled < 0) {
        const char* e = getenv("TSM_IGEMM_NARROW");
        enabled = (e && e[0] == '0') ? 0 : 1;
    }
    if (!enabled || ring_rows(rows, Cd) != 128) return 128;
    const long tiles = ((rows + 127) / 128) * ((Cd + 127) / 128);
    return tiles * 4 < (long)num_cu() * 3 ? 64 : 128;
}

// Tile of the ring kernel for a layer (one block per CU whatever the tile: the 128 x 64 tile with two blocks per CU,
// tried on the 1x1 data gradients with one to eight K steps so that one block's epilogue overlaps the other's main
// loop, was 3 - 20 % slower on them than 256 x 128 tiles).
static void ring_tile(const IgemmArgs& a, int* bm, int* bn) {
    const long rows = (long)a.F * a.Hd * a.Wd;
    *bm = ring_rows(rows, a.Cd);
    *bn = ring_cols(rows, a.Cd);
}

// The 64 -> 64 channel 3x3 kernel takes the layers it is written for when the general kernel would run them with
// 256-row tiles (the two then launch the same number of blocks, which is what callers size the statistics rows by)
// and there are at least five rounds of tiles: every block first loads all weights and a tile is long, so with
// three rounds (8 clips) the general kernel is 1 % of the step faster, with six (16 clips) the two are level, with
// 24 (64 clips) this one saves 1.1 % of the step.  TSM_CONV3X3_C64=0 leaves these layers to the general kernel,
// TSM_CONV3X3_C64_MIN_TILES=<n> moves the threshold (both read at every call: tests and comparisons set them).
static bool c64_eligible(const IgemmArgs& a) {
    const char* e = getenv("TSM_CONV3X3_C64");
    const bool enabled = !(e && e[0] == '0');
    const char* t = getenv("TSM_CONV3X3_C64_MIN_TILES");
    const long min_tiles = t ? atol(t) : 5L * num_cu();
    const long rows = (long)a.F * a.Hd * a.Wd;
    return enabled && (rows + C64_BM - 1) / C64_BM >= min_tiles && a.Cs == 64 && a.Cd == 64 && a.pitch == 64 && a.KT == 1 && a.KH == 3 && a.KW == 3 && a.stride == 1 &&
           a.padh == 1 && a.padw == 1 && a.fold == 0 && a.addend == nullptr && a.Hs == a.Hd && a.Ws == a.Wd &&
           a.Ws <= C64_WMAX && (rows + a.Ws + 1) * 128 < 0x7ff00000L &&
           ring_eligible(64, rows * 64 + 64 + (long)(a.Ws + 1) * 64, 64L * a.K, false) && ring_rows(rows, 64) == 256;
}

template <bool DGRAD, bool STREAM>
static int launch_c64_s(IgemmArgs& a, hipStream_t s) {
    auto kern = conv3x3_c64_kernel<DGRAD, STREAM>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "conv3x3_c64: cannot raise dynamic LDS limit");
        configured = true;
    }
    const long rows = (long)a.F * a.Hd * a.Wd;
    const int grid = igemm_grid((int)((rows + C64_BM - 1) / C64_BM), 64, 64, 1);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), C64_SMEM, s, a);
    return check_launch(DGRAD ? "igemm_dgrad_c64" : "igemm_fwd_c64");
}

template <bool DGRAD>
static int launch_c64(IgemmArgs& a, hipStream_t s) {
    if ((long)a.F * a.Hd * a.Wd * a.Cd * 2 > (64L << 20)) return launch_c64_s<DGRAD, true>(a, s);
    return launch_c64_s<DGRAD, false>(a, s);
}

// ---------------------------------------------------------------------------------
// The stem in space-to-depth form, forward with the statistics epilogue, one wavefront per 32 output pixels (the scheme
// of pw_fwd_kernel): the layer writes 128 bytes per output pixel and reads a fifth of that, so it is a stream of stores
// with a product attached (K = 256: 32 MFMAs per pass), and in the block-wide schedule of stem_s2d_kernel the eight
// wavefronts wait on each other between the patch, the product and the two epilogue passes.  Here the weights (32 KB)
// sit in LDS for the life of the block; a wavefront reads the sixteen 16-byte fragments of its pixels straight from
// memory (tap row th, pixel ks of the row's four, half lane / 32: neighbouring output pixels share three of their four
// input pixels per row, which the caches serve), multiplies, passes the 32 x 64 result through a staging tile of its
// own and stores 128 contiguous bytes per pixel; the next pass's fragments are requested before this pass is
// multiplied.  No block barrier in the loop.  Partial rows (a.stats): one per block, [2][64].
static constexpr int SPW_LDC = 64 + 8;
static constexpr int SPW_CST_BYTES = 32 * SPW_LDC * 2;        // per wavefront
static constexpr int SPW_SMEM = STEM_W_BYTES + 8 * SPW_CST_BYTES + 2 * 8 * 64 * 4;

template <bool STREAM>
__global__ void __launch_bounds__(512) stem_pw_kernel(IgemmArgs a) {
    constexpr int LDC = SPW_LDC;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* s_w = smem;                                                       // [4][64][8 positions of 16 bytes], swizzled
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bf16_t* Cst = (bf16_t*)(smem + STEM_W_BYTES + wave * SPW_CST_BYTES);             // [32][LDC], this wavefront's
    float* s_part = (float*)(smem + STEM_W_BYTES + 8 * SPW_CST_BYTES);               // [2 stats][8 wavefronts][64]
    const int r = lane & 31, hi = lane >> 5;
    const int Ws = a.Ws, Wd = a.Wd, hw_d = a.Hd * a.Wd, hw_s = a.Hs * a.Ws;
    const unsigned M = (unsigned)a.F * (unsigned)hw_d;            // output pixels
    const unsigned Min = (unsigned)a.F * (unsigned)hw_s;          // input pixels
    const bool do_stats = a.stats != nullptr;

    {
        const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(a.wp, (uint32_t)(64 * 256 * 2));
#pragma unroll
        for (int sidx = 0; sidx < 4; ++sidx) {
            const int q = tid + sidx * 512;                       // piece: tap row sidx, channel row n, position pos
            const int n = (q >> 3) & 63, pos = q & 7, kv = pos ^ ((n >> 1) & 7);
            *(u32x4*)(s_w + q * 16) = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, n * 512 + sidx * 128 + kv * 16, 0, 0);
        }
    }
    __syncthreads();

    int b_rd[4];                                                   // fragment of weight rows 32*j + r, step ks of a tap row
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) b_rd[ks] = r * 128 + (((2 * ks + hi) ^ ((r >> 1) & 7)) * 16);
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(a.src, (uint32_t)((long)Min * 32));
    const unsigned nslabs = (M + 31) / 32;
    const unsigned nwaves = gridDim.x * 8;
    bf16x8 cur[16], nxt[16];
    auto load_a = [&](unsigned sl, bf16x8* fr) {
        const unsigned P = sl * 32 + (unsigned)r;
        unsigned base = OOB_OFFSET;
        if (P < M) {
            const unsigned f = P / (unsigned)hw_d, q = P - f * (unsigned)hw_d;
            const unsigned h = q / (unsigned)Wd, w = q - h * (unsigned)Wd;
            base = (f * (unsigned)hw_s + h * (unsigned)Ws + w) * 32u + (unsigned)hi * 16u;
        }
#pragma unroll
        for (int th = 0; th < 4; ++th)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, P < M ? (int)(base + (unsigned)(th * Ws + ks) * 32u) : (int)OOB_OFFSET, 0, 0);
                fr[th * 4 + ks] = __builtin_bit_cast(bf16x8, v);
            }
    };
    float f1[8], f2[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) f1[q] = f2[q] = 0.f;
    const int vcol = lane & 7, row0 = lane >> 3;                   // store loop: piece lane + 64*t is row row0 + 8*t, vector vcol

    unsigned slab = blockIdx.x * 8 + (unsigned)wave;
    if (slab < nslabs) load_a(slab, cur);
    for (; slab < nslabs; slab += nwaves) {
        if (slab + nwaves < nslabs) load_a(slab + nwaves, nxt);    // in flight while this pass is multiplied and stored
        f32x16 acc[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
#pragma unroll
        for (int th = 0; th < 4; ++th)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bf16x8 bfrag = *(const bf16x8*)(s_w + th * (64 * 128) + j * 32 * 128 + b_rd[ks]);
                    // operands swapped as in igemm_ring_kernel: the result block is [channel][pixel]
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, cur[th * 4 + ks], acc[j], 0, 0, 0);
                }
        // lane: pixel r, channels 32*j + 8*q + 4*hi + {0..3}
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            bf16_t* dstp = Cst + r * LDC + j * 32 + 4 * hi;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint2 w;
                w.x = pack_bf16x2(acc[j][4 * q], acc[j][4 * q + 1]);
                w.y = pack_bf16x2(acc[j][4 * q + 2], acc[j][4 * q + 3]);
                *(uint2*)(dstp + 8 * q) = w;
            }
        }
        __builtin_amdgcn_wave_barrier();                           // (LDS serves a wavefront's accesses in order)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = row0 + 8 * t;
            const unsigned P = slab * 32 + (unsigned)row;
            const u32x4 v = *(const u32x4*)(Cst + row * LDC + vcol * 8);
            if (P < M) {
                if (do_stats) {   // statistics of the values as stored
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(v[e] << 16), hv = __uint_as_float(v[e] & 0xffff0000u);
                        f1[2 * e] += lo;
                        f1[2 * e + 1] += hv;
                        f2[2 * e] = fmaf(lo, lo, f2[2 * e]);
                        f2[2 * e + 1] = fmaf(hv, hv, f2[2 * e + 1]);
                    }
                }
                u32x4* q = (u32x4*)(a.dst + (long)P * 64 + vcol * 8);
                if (STREAM) __builtin_nontemporal_store(v, q);
                else *q = v;
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < 16; ++q) cur[q] = nxt[q];
    }
    if (do_stats) {
        // lanes 8 apart hold the same columns: fold them, then one slot per wavefront, fixed order over the slots
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int off = 8; off < 64; off <<= 1) {
                f1[q] += __shfl_xor(f1[q], off);
                f2[q] += __shfl_xor(f2[q], off);
            }
        if (lane < 8) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                s_part[wave * 64 + lane * 8 + q] = f1[q];
                s_part[(8 + wave) * 64 + lane * 8 + q] = f2[q];
            }
        }
        __syncthreads();
        if (tid < 128) {
            const int stat = tid >> 6, c = tid & 63;
            float v = 0.f;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) v += s_part[(stat * 8 + sl) * 64 + c];
            a.stats[((size_t)blockIdx.x * 2 + stat) * 64 + c] = v;
        }
    }
}

// The stem kernel: the space-to-depth stem (forward), under the same conditions as the 64-channel 3x3 kernel and
// the same switches; the worst-case patch of a tile (output rows crossed, a frame boundary crossed) must fit.
static bool stem_eligible(const IgemmArgs& a) {
    const char* e = getenv("TSM_CONV3X3_C64");
    const char* e2 = getenv("TSM_STEM_KERNEL");
    const bool enabled = !(e && e[0] == '0') && !(e2 && e2[0] == '0');
    const char* t = getenv("TSM_CONV3X3_C64_MIN_TILES");
    const long min_tiles = t ? atol(t) : 5L * num_cu();
    const long rows = (long)a.F * a.Hd * a.Wd;
    if (!(enabled && a.Cs == 64 && a.Cd == 64 && a.pitch == 16 && a.KT == 1 && a.KH == 4 && a.KW == 1 && a.stride == 1 &&
          a.padh == 0 && a.padw == 0 && a.fold == 0 && a.addend == nullptr && a.Hd == a.Hs - 3 && a.Wd == a.Ws - 3 && a.Wd >= 1 &&
          a.Hd >= 1))
        return false;
    // A tile's patch runs from the first output pixel's window to the end of the last one's: the input rows under the
    // output rows it crosses, three more per frame boundary it crosses, the three tap rows below, and less than a row.
    const long hw_d = (long)a.Hd * a.Wd;
    const long rows_crossed = (STEM_BM - 1) / a.Wd + 1, frames_crossed = (STEM_BM - 1) / hw_d + 1;
    const long worst = (rows_crossed + 3 * frames_crossed) * a.Ws + (a.Wd - 1) + 3L * a.Ws + 4;
    return worst <= STEM_PMAX && (rows + STEM_BM - 1) / STEM_BM >= min_tiles && (long)a.F * a.Hs * a.Ws * 32 < 0x7ff00000L &&
           ring_eligible(64, (long)a.F * a.Hs * a.Ws * 16 + 64, 64L * a.K, true) && ring_rows(rows, 64) == 256;
}

// (the wavefront-per-32-pixels variant takes the stem wherever no affine epilogue is asked for -- it carries the
//  statistics epilogue only; TSM_STEM_PW=0, read at every call, keeps the block-wide kernel)
template <bool STREAM>
static int launch_stem_pw(IgemmArgs& a, hipStream_t s) {
    auto kern = stem_pw_kernel<STREAM>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "stem_pw: cannot raise dynamic LDS limit");
        configured = true;
    }
    const long rows = (long)a.F * a.Hd * a.Wd;
    const int grid = igemm_grid((int)((rows + STEM_BM - 1) / STEM_BM), 64, 64, 1);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), SPW_SMEM, s, a);
    return check_launch("igemm_fwd_stem");
}

template <bool STREAM>
static int launch_stem_s(IgemmArgs& a, hipStream_t s) {
    auto kern = stem_s2d_kernel<STREAM>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "stem_s2d: cannot raise dynamic LDS limit");
        configured = true;
    }
    const long rows = (long)a.F * a.Hd * a.Wd;
    const int grid = igemm_grid((int)((rows + STEM_BM - 1) / STEM_BM), 64, 64, 1);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), STEM_SMEM, s, a);
    return check_launch("igemm_fwd_stem");
}

// The short-K 1x1 forward kernel takes its layers when the general kernel would run them with 256-row tiles (the two
// then launch the same number of blocks, which callers size the statistics rows by) and every wavefront of the grid has
// a pass of its own (measured at 8 clips: 6.92 -> 6.83 ms against a threshold of two passes).  TSM_PW_KERNEL=0 leaves
// these layers to the general kernel, TSM_PW_MIN_ROWS=<n> moves the threshold (both read at every call: tests and
// comparisons set them).
// (K = 64, 128: a block holds 256 result channels; K = 256: 128.  The threshold counts the passes of the streams that
// the grid forms.)
static int pw_block_channels(int Cs) { return Cs <= 128 ? 256 : 128; }
static bool pw_shape_ok(const IgemmArgs& a) {
    const char* e = getenv("TSM_PW_KERNEL");
    if (e && e[0] == '0') return false;
    if (!((a.Cs == 64 || a.Cs == 128 || a.Cs == 256) && a.pitch == a.Cs && a.KT == 1 && a.KH == 1 && a.KW == 1 && a.stride == 1 &&
          a.padh == 0 && a.padw == 0 && a.Hs == a.Hd && a.Ws == a.Wd))
        return false;
    const int nb = pw_block_channels(a.Cs);
    if (a.Cd < 256 || a.Cd > 1024 || a.Cd % nb != 0 || a.Cd < 2 * a.Cs) return false;     // wide results only
    const long rows = (long)a.F * a.Hd * a.Wd;
    const char* t = getenv("TSM_PW_MIN_ROWS");
    const long min_rows = t ? atol(t) : 32L * 8 * num_cu() / (a.Cd / nb);
    return rows <= 0x7fffffffL && rows * a.Cs * 2 < 0x7ff00000L && ring_eligible(a.Cs, rows * a.Cs + a.Cs, (long)a.Cd * a.Cs, false) &&
           ring_rows(rows, a.Cd) == 256 && rows >= min_rows;
}

static bool pw_fwd_eligible(const IgemmArgs& a) {
    // (the affine epilogue: variants for K = 64 and K = 256, the inference call's layers outside its fused kernels)
    return pw_shape_ok(a) && a.fold == 0 && a.addend == nullptr && (a.ep_scale == nullptr || a.Cs != 128);
}

template <int KC, bool STREAM, bool AFF = false>
static int launch_pw_fwd(IgemmArgs& a, hipStream_t s) {
    auto kern = pw_fwd_kernel<KC, STREAM, AFF>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "pw_fwd: cannot raise dynamic LDS limit");
        configured = true;
    }
    const long rows = (long)a.F * a.Hd * a.Wd;
    const int grid = igemm_grid((int)((rows + 255) / 256), a.Cd, 128, 1);      // as the general kernel with 256 x 128 tiles
    if (grid % (a.Cd / PwD<KC>::NB) != 0) return fail(TSM_ERR_LAUNCH, "pw_fwd: grid does not split over the parts of the result");
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), PwD<KC>::SMEM, s, a);
    return check_launch("igemm_fwd_pw");
}

// The short-K, wide-result 1x1 data-gradient kernel takes its layers under the same conditions as the forward kernel
// above; where the epilogue needs a ReLU mask, only with the decision bits (see DgradFuse::act_bits).
static bool pw_dgrad_eligible(const IgemmArgs& a) {
    if (!pw_shape_ok(a) || a.fold % 8 != 0) return false;
    if (a.add_stride == 2 && !(a.addend != nullptr && a.Cs >= 128)) return false;   // the compact addend: variants for K = 128, 256
    if (a.act != nullptr && a.act_bits == nullptr) return false;      // a mask that only the activation can give
    if (a.ybn != nullptr && a.stats == nullptr) return false;
    return true;
}

template <int KC, bool STREAM, bool CADD = false>
static int launch_pw_dgrad(IgemmArgs& a, hipStream_t s) {
    auto kern = pw_dgrad_kernel<KC, STREAM, CADD>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "pw_dgrad: cannot raise dynamic LDS limit");
        configured = true;
    }
    const long rows = (long)a.F * a.Hd * a.Wd;
    const int grid = igemm_grid((int)((rows + 255) / 256), a.Cd, 128, 1);      // as the general kernel with 256 x 128 tiles
    if (grid % (a.Cd / PwD<KC>::NB) != 0) return fail(TSM_ERR_LAUNCH, "pw_dgrad: grid does not split over the parts of the result");
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), PwD<KC>::SMEM, s, a);
    return check_launch("igemm_dgrad_pw");
}

// Forward layers whose result is a multiple of 256 channels wide take 256 x 256 tiles (wavefront tiles of 128 x 64:
// three quarters of the LDS fragment bytes and two thirds of the operand stream per MFMA of the 256 x 128 tile) when
// the general kernel would run them with 256-row tiles, no kernel of their own takes them, they have no affine
// epilogue (the variant keeps the statistics epilogue only) and the wide tiles still give half of the CUs a tile
// (measured: better from 148 tiles on, worse at 98).  TSM_IGEMM_WIDE=0 (read at every call) keeps 128 columns, TSM_IGEMM_WIDE_MIN_TILES=<n> replaces the number
// of wide tiles from which they are chosen (tests and comparisons set them).
static bool wide_fwd_eligible(const IgemmArgs& a) {
    const char* e = getenv("TSM_IGEMM_WIDE");
    if (e && e[0] == '0') return false;
    const char* t = getenv("TSM_IGEMM_WIDE_MIN_TILES");
    const long min_tiles = t ? atol(t) : ((long)num_cu() + 1) / 2;
    const long rows = (long)a.F * a.Hd * a.Wd;
    if (a.Cd % 256 != 0 || a.ep_scale != nullptr || a.addend != nullptr || a.pitch != a.Cs) return false;
    if (pw_fwd_eligible(a)) return false;
    if (!ring_eligible(a.Cs, (long)a.F * a.Hs * a.Ws * a.pitch + a.Cs + (long)(a.padh * a.Ws + a.padw) * a.pitch, (long)a.Cd * a.K, false)) return false;
    if (ring_rows(rows, a.Cd) != 256) return false;
    return ((rows + 255) / 256) * (a.Cd / 256) >= min_tiles;
}

template <bool DGRAD>
static int dispatch_igemm(IgemmArgs& a, hipStream_t s) {
    const long rows = (long)a.F * a.Hd * a.Wd;
    if (rows == 0) return TSM_OK;
    if (c64_eligible(a)) return launch_c64<DGRAD>(a, s);
    if (DGRAD && pw_dgrad_eligible(a)) {
        const bool st = rows * a.Cd * 2 > (64L << 20);
        if (a.Cs == 64) return st ? launch_pw_dgrad<64, true>(a, s) : launch_pw_dgrad<64, false>(a, s);
        if (a.Cs == 128) {
            if (a.add_stride == 2) return st ? launch_pw_dgrad<128, true, true>(a, s) : launch_pw_dgrad<128, false, true>(a, s);
            return st ? launch_pw_dgrad<128, true>(a, s) : launch_pw_dgrad<128, false>(a, s);
        }
        if (a.add_stride == 2) return st ? launch_pw_dgrad<256, true, true>(a, s) : launch_pw_dgrad<256, false, true>(a, s);
        return st ? launch_pw_dgrad<256, true>(a, s) : launch_pw_dgrad<256, false>(a, s);
    }
    if (!DGRAD && pw_fwd_eligible(a)) {
        const bool st = rows * a.Cd * 2 > (64L << 20);
        if (a.ep_scale != nullptr) {   // the affine epilogue of the inference path
            if (a.Cs == 64) return st ? launch_pw_fwd<64, true, true>(a, s) : launch_pw_fwd<64, false, true>(a, s);
            return st ? launch_pw_fwd<256, true, true>(a, s) : launch_pw_fwd<256, false, true>(a, s);
        }
        if (a.Cs == 64) return st ? launch_pw_fwd<64, true>(a, s) : launch_pw_fwd<64, false>(a, s);
        if (a.Cs == 128) return st ? launch_pw_fwd<128, true>(a, s) : launch_pw_fwd<128, false>(a, s);
        return st ? launch_pw_fwd<256, true>(a, s) : launch_pw_fwd<256, false>(a, s);
    }
    if (!DGRAD && stem_eligible(a)) {
        const char* pe = getenv("TSM_STEM_PW");
        if (a.ep_scale == nullptr && rows < 0x7fffffffL / 2 && !(pe && pe[0] == '0'))
            return rows * a.Cd * 2 > (64L << 20) ? launch_stem_pw<true>(a, s) : launch_stem_pw<false>(a, s);
        return rows * a.Cd * 2 > (64L << 20) ? launch_stem_s<true>(a, s) : launch_stem_s<false>(a, s);
    }
    if (ring_eligible(a.Cs, (long)a.F * a.Hs * a.Ws * a.pitch + a.Cs + (long)(a.padh * a.Ws + a.padw) * a.pitch, (long)a.Cd * a.K, a.pitch != a.Cs)) {
        if constexpr (!DGRAD) {
            if (wide_fwd_eligible(a)) return launch_igemm_ring<256, 256, 2, 4, false>(a, "igemm_fwd_256x256", s);
        }
        int bm, bn;
        ring_tile(a, &bm, &bn);
        if (bm == 128) {
            if (bn == 64) return launch_igemm_ring<128, 64, 4, 2, DGRAD>(a, DGRAD ? "igemm_dgrad_r128x64" : "igemm_fwd_r128x64", s);
            return launch_igemm_ring<128, 128, 4, 2, DGRAD>(a, DGRAD ? "igemm_dgrad_r128x128" : "igemm_fwd_r128x128", s);
        }
        if (a.Cd <= 64) return launch_igemm_ring<256, 64, 4, 2, DGRAD>(a, DGRAD ? "igemm_dgrad_256x64" : "igemm_fwd_256x64", s);
        return launch_igemm_ring<256, 128, 4, 2, DGRAD>(a, DGRAD ? "igemm_dgrad_256x128" : "igemm_fwd_256x128", s);
    }
    if (a.pitch != a.Cs) return fail(TSM_ERR_UNSUPPORTED, "igemm: a pixel pitch other than the channel count needs the 64-channel-step kernel");
    if (a.Cd <= 64) return launch_igemm<128, 64, 4, 1, DGRAD, 1, 2>(a, DGRAD ? "igemm_dgrad_128x64" : "igemm_fwd_128x64", s);
    return launch_igemm<128, 128, 2, 2, DGRAD, 1, 2>(a, DGRAD ? "igemm_dgrad_128x128" : "igemm_fwd_128x128", s);
}

static void fwd_args(const ConvP& p, IgemmArgs& a) {
    a.F = p.F; a.T = p.T;
    a.Hs = p.H; a.Ws = p.W; a.Cs = p.Cin; a.pitch = p.pix_pitch();
    a.Hd = p.Ho; a.Wd = p.Wo; a.Cd = p.Cout;
    a.KT = p.KT; a.KH = p.KH; a.KW = p.KW;
    a.stride = p.stride; a.padh = p.pad; a.padw = p.pad;
    a.fold = p.fold;
    a.K = (int)p.K();
}

// Blocks the forward convolution with the statistics epilogue launches (= partial rows it writes).
int conv_mfma_fwd_blocks(const ConvP& p) {
    const int bn = p.Cout <= 64 ? 64 : 128;
    {
        IgemmArgs a;
        a.addend = nullptr; a.ep_scale = nullptr;
        fwd_args(p, a);
        if (wide_fwd_eligible(a)) return igemm_grid((int)((p.rows_out() + 255) / 256), p.Cout, 256, 1);
    }
    if (ring_eligible(p.Cin, p.rows_in() * (long)p.pix_pitch() + p.Cin + (long)(p.pad * p.W + p.pad) * p.pix_pitch(), (long)p.Cout * p.K(), p.pix_pitch() != p.Cin))
    {
        const int bm = ring_rows(p.rows_out(), p.Cout), bnn = ring_cols(p.rows_out(), p.Cout);
        return igemm_grid((int)((p.rows_out() + bm - 1) / bm), p.Cout, bnn, 1);
    }
    return igemm_grid((int)((p.rows_out() + 127) / 128), p.Cout, bn, 2);
}

bool conv_mfma_fwd_can_fuse(const ConvP& p) {
    return ring_eligible(p.Cin, p.rows_in() * (long)p.pix_pitch() + p.Cin + (long)(p.pad * p.W + p.pad) * p.pix_pitch(), (long)p.Cout * p.K(),
                         p.pix_pitch() != p.Cin);
}

int conv_mfma_fwd(const ConvP& p, const bf16_t* x, const bf16_t* wp, bf16_t* y, float* stats, const FwdEpilogue* ep,
                  hipStream_t s) {
    IgemmArgs a;
    a.src = x; a.wp = wp; a.dst = y; a.addend = nullptr; a.add_stride = 1; a.add_ho = a.add_wo = 0; a.stats = stats;
    a.act = nullptr; a.ybn = nullptr; a.bn_mean = nullptr; a.bn_rstd = nullptr; a.act_bits = nullptr;
    a.ep_scale = nullptr; a.ep_shift = nullptr; a.ep_res = nullptr; a.ep_relu = 0;
    if (ep) {
        if (!conv_mfma_fwd_can_fuse(p)) return fail(TSM_ERR_UNSUPPORTED, "conv forward: this layer's kernel has no affine epilogue");
        a.ep_scale = ep->scale; a.ep_shift = ep->shift; a.ep_res = ep->res; a.ep_relu = ep->relu;
    }
    fwd_args(p, a);
    return dispatch_igemm<false>(a, s);
}

static void dgrad_args(const ConvP& p, IgemmArgs& a) {
    a.F = p.F; a.T = p.T;
    a.Hs = p.Ho; a.Ws = p.Wo; a.Cs = p.Cout; a.pitch = p.Cout;
    a.Hd = p.H; a.Wd = p.W; a.Cd = p.Cin;
    a.KT = p.KT; a.KH = p.KH; a.KW = p.KW;
    a.stride = p.stride; a.padh = p.KH - 1 - p.pad; a.padw = p.KW - 1 - p.pad;
    a.fold = p.fold;
    a.K = p.taps() * p.Cout;
}

int conv_mfma_dgrad_blocks(const ConvP& p) {
    IgemmArgs a;
    dgrad_args(p, a);
    if (!ring_eligible(a.Cs, (long)a.F * a.Hs * a.Ws * a.pitch + a.Cs + (long)(a.padh * a.Ws + a.padw) * a.pitch, (long)a.Cd * a.K, a.pitch != a.Cs)) return 0;
    if ((long)a.F * a.Hd * a.Wd == 0) return 0;
    int bm, bn;
    ring_tile(a, &bm, &bn);
    const int mtiles = setup_classes(a, true, bm);
    return igemm_grid(mtiles, a.Cd, bn, 1);
}

bool conv_mfma_dgrad_compact_addend_ok(const ConvP& p) { return conv_mfma_dgrad_blocks(p) > 0; }

int conv_mfma_dgrad(const ConvP& p, const bf16_t* dy, const bf16_t* wd, bf16_t* dx, const bf16_t* addend,
                    const DgradFuse* fuse, hipStream_t s, int addend_stride) {
    IgemmArgs a;
    a.src = dy; a.wp = wd; a.dst = dx; a.addend = addend; a.stats = nullptr;
    a.add_stride = 1; a.add_ho = a.add_wo = 0;
    if (addend && addend_stride != 1) {
        if (addend_stride != 2 || !conv_mfma_dgrad_compact_addend_ok(p))
            return fail(TSM_ERR_UNSUPPORTED, "dgrad: this layer's kernel takes a dense addend only");
        a.add_stride = 2; a.add_ho = (p.H + 1) / 2; a.add_wo = (p.W + 1) / 2;
    }
    a.act = nullptr; a.ybn = nullptr; a.bn_mean = nullptr; a.bn_rstd = nullptr; a.act_bits = nullptr;
    a.ep_scale = nullptr; a.ep_shift = nullptr; a.ep_res = nullptr; a.ep_relu = 0;
    dgrad_args(p, a);
    if (fuse) {
        // (the general kernel reads the decision bits where it has them; the 64-channel kernel and tiles without the
        // variant read `act`)
        static int bits_on = -1;   // TSM_MASK_BITS=0 keeps the activation as the mask source (for comparisons)
        if (bits_on < 0) {
            const char* e = getenv("TSM_MASK_BITS");
            bits_on = (e && e[0] == '0') ? 0 : 1;
        }
        if (bits_on && p.Cin % 8 == 0) a.act_bits = fuse->act_bits;
        if (conv_mfma_dgrad_blocks(p) == 0) return fail(TSM_ERR_UNSUPPORTED, "dgrad: this layer's kernel cannot fuse the BatchNorm reductions");
        // (y == nullptr: only the ReLU mask of `act` is applied, no sums)
        a.act = fuse->act; a.ybn = fuse->y; a.bn_mean = fuse->mean; a.bn_rstd = fuse->rstd; a.stats = fuse->y ? fuse->partial : nullptr;
    }
    return dispatch_igemm<true>(a, s);
}

// ---------------------------------------------------------------------------------
// Weight gradient, D[Cout x K] = dy^T [Cout x pixels] * gathered x [pixels x K] with
// K = taps * Cin enumerated tap-major (the packed-weight order).  Per block: a
// [BCO x BCI] tile of D reduced over a chunk of output pixels, added with fp32
// atomics to dw.  Both MFMA operands are needed with the pixel index contiguous, so
// the 16-byte global rows ([pixel][channel]) are transposed on their way into LDS:
// each thread takes four consecutive pixels of eight channels and writes, per
// channel, the four pixels as one 64-bit LDS store.
struct WgradArgs {
    const bf16_t* x;
    const bf16_t* dy;
    float* dw;             // element (co, ci, tap) at co*so + ci*si + tap*st
    long so;
    int si, st, cin_real;
    int F, T;
    int H, W, Cin;
    int pitch;             // elements between consecutive input pixels (Cin, or less: see ConvP::pitch)
    int Ho, Wo, Cout;
    int KT, KH, KW, stride, pad;
    int fold;
    long M;                // output pixels
    long chunk;            // pixels per block (multiple of 64)
    int K;                 // taps * Cin
    int col_tiles;
    int tiles, nchunks, group;   // wgrad_tr_kernel: tiles of D, chunks of pixels, block index mapping (see the kernel)
    // wgrad_tr_kernel, AFF variants: dy is not stored; the loader forms it from dz (passed as `dy`) and the
    // BatchNorm input ay as dy = a*dz + b*ay + c per output channel, coefficients aff = [3][Cout] (BatchNorm
    // backward, see bn_bwd_apply), rounded to bf16 as the stored tensor would be
    const bf16_t* ay;
    const float* aff;
};

static constexpr int WMK = 64;        // pixels per main-loop step
static constexpr int LDT = WMK + 8;   // pitch of the transposed tiles

// Transposed-tile rows are [channel][pixel] with a 144-byte pitch.  The transposing 8-byte stores come
// from lanes whose rows are 8 apart, which would all fall into the same banks; the 16-byte pixel groups of
// a row are therefore XOR-ed with the row's channel-vector index (measured faster than leaving the groups
// in place or XOR-ing with a coarser row index).
__device__ __forceinline__ int swz_x(int row) { return (row >> 3) & 7; }
// Element offset of pixel quad `pq` (four pixels = 8 bytes) in row `row`.
__device__ __forceinline__ int swz_quad(int pq, int row) { return (((pq >> 1) ^ swz_x(row)) << 3) | ((pq & 1) << 2); }
// Element offset of the 8-pixel fragment `g` (0..7) of row `row`.
__device__ __forceinline__ int swz_frag(int g, int row) { return (g ^ swz_x(row)) * 8; }

template <int BCO, int BCI>
__global__ void __launch_bounds__(256, 2) wgrad_kernel(WgradArgs a) {
    constexpr int TM = BCO / 2, TN = BCI / 2;
    constexpr int MI = TM / 32, NJ = TN / 32;
    constexpr int AV = BCO / 8, BV = BCI / 8;         // 16-byte vectors per tile row
    constexpr int AITEMS = AV * (WMK / 4), BITEMS = BV * (WMK / 4);   // (vector, pixel quad) work items
    static_assert(AITEMS <= 256, "one dy item per thread");
    constexpr int BQ = (BITEMS + 255) / 256;                          // x items per thread
    __shared__ __attribute__((aligned(16))) bf16_t At[2][BCO][LDT];   // dy^T  [co][pixel]
    __shared__ __attribute__((aligned(16))) bf16_t Bt[2][BCI][LDT];   // xs^T  [column][pixel]
    __shared__ RowInfo s_info[3][WMK];                                // per-pixel gather origin, three steps deep

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int co0 = (blockIdx.y / a.col_tiles) * BCO;
    const int j0 = (blockIdx.y % a.col_tiles) * BCI;
    const long mbeg = (long)blockIdx.x * a.chunk;
    long mend = mbeg + a.chunk;
    if (mend > a.M) mend = a.M;
    if (mbeg >= mend) return;
    const int hw = a.Ho * a.Wo;
    const bf16_t* zero_page = (const bf16_t*)g_zero_page;

    // ---- this thread's work items: consecutive lanes take consecutive 16-byte pieces of a pixel row
    const int avec = tid % AV, apq = tid / AV;        // dy: channels co0 + 8*avec.., pixels 4*apq..4*apq+3
    const bool a_item = tid < AITEMS;
    const bool a_chan_ok = co0 + avec * 8 < a.Cout;
    // x items: columns j0 + 8*bvec.., pixel quad bpq; column -> (tap, channel) is constant for the thread's life
    int bvec[BQ], bpq[BQ], boff[BQ];
    uint32_t need[BQ];
    bool b_item[BQ];
#pragma unroll
    for (int q = 0; q < BQ; ++q) {
        const int item = q * 256 + tid;
        bvec[q] = item % BV;
        bpq[q] = item / BV;
        b_item[q] = item < BITEMS;
        need[q] = 0xffffffffu;   // unsatisfiable: column beyond K
        boff[q] = 0;
        const int j = j0 + bvec[q] * 8;
        if (j < a.K) {
            const int tap = j / a.Cin, ci = j - tap * a.Cin;
            const int kw = tap % a.KW, kh = (tap / a.KW) % a.KH, kt = tap / (a.KW * a.KH);
            const int d = kt - a.KT / 2 + group_dt(ci, a.fold);
            need[q] = (1u << kh) | (1u << (8 + kw)) | (d > 0 ? 1u << 30 : 0u) | (d < 0 ? 1u << 31 : 0u);
            boff[q] = d * a.H * a.W * a.Cin + (kh * a.W + kw) * a.Cin + ci;
        }
    }

    // ---- per-step decode of the 64 pixels' gather origins (one pixel per thread of the first wavefront)
    auto decode = [&](int st) {
        if (tid < WMK) {
            const long m = mbeg + (long)st * WMK + tid;
            RowInfo info;
            info.off = 0;
            info.mask = 0;
            info.dst = 0;
            if (m < mend) {
                const int f = (int)(m / hw);
                const int pix = (int)(m - (long)f * hw);
                const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
                const int ih = oh * a.stride - a.pad, iw = ow * a.stride - a.pad;
                const int t = f % a.T;
                uint32_t mask = 0;
                for (int kh = 0; kh < a.KH; ++kh)
                    if (ih + kh >= 0 && ih + kh < a.H) mask |= 1u << kh;
                for (int kw = 0; kw < a.KW; ++kw)
                    if (iw + kw >= 0 && iw + kw < a.W) mask |= 1u << (8 + kw);
                if (t + 1 < a.T) mask |= 1u << 30;
                if (t >= 1) mask |= 1u << 31;
                info.off = ((long)f * a.H * a.W + (long)ih * a.W + iw) * a.Cin;
                info.mask = mask;
            }
            s_info[st % 3][tid] = info;
        }
    };

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 ar[4], br[BQ][4];

    auto load = [&](int st) {
        const long mstep = mbeg + (long)st * WMK;
        if (a_item) {
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const long m = mstep + 4 * apq + h;
                const bf16_t* p = (a_chan_ok && m < mend) ? a.dy + m * a.Cout + co0 + avec * 8 : zero_page;
                ar[h] = *(const u32x4*)p;
            }
        }
#pragma unroll
        for (int q = 0; q < BQ; ++q) {
            if (b_item[q]) {
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const RowInfo ri = s_info[st % 3][4 * bpq[q] + h];
                    const bf16_t* p = ((ri.mask & need[q]) == need[q]) ? a.x + ri.off + boff[q] : zero_page;
                    br[q][h] = *(const u32x4*)p;
                }
            }
        }
    };
    // four pixels x eight channels -> per channel one 8-byte store of four pixels
    auto scatter = [&](bf16_t (*Tt)[LDT], int vec, int pq, const u32x4* v) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint2 even, odd;
            even.x = __builtin_amdgcn_perm(v[1][e], v[0][e], 0x05040100u);
            even.y = __builtin_amdgcn_perm(v[3][e], v[2][e], 0x05040100u);
            odd.x = __builtin_amdgcn_perm(v[1][e], v[0][e], 0x07060302u);
            odd.y = __builtin_amdgcn_perm(v[3][e], v[2][e], 0x07060302u);
            *(uint2*)&Tt[vec * 8 + 2 * e][swz_quad(pq, vec * 8)] = even;
            *(uint2*)&Tt[vec * 8 + 2 * e + 1][swz_quad(pq, vec * 8)] = odd;
        }
    };
    auto store = [&](int buf) {
        if (a_item) scatter(At[buf], avec, apq, ar);
#pragma unroll
        for (int q = 0; q < BQ; ++q)
            if (b_item[q]) scatter(Bt[buf], bvec[q], bpq[q], br[q]);
    };

    const int nsteps = (int)((mend - mbeg + WMK - 1) / WMK);
    decode(0);
    if (nsteps > 1) decode(1);
    __syncthreads();
    load(0);
    store(0);
    __syncthreads();
    for (int st = 0; st < nsteps; ++st) {
        const int buf = st & 1;
        if (st + 2 < nsteps) decode(st + 2);
        if (st + 1 < nsteps) load(st + 1);
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

// ---------------------------------------------------------------------------------
// Weight gradient for input channel counts that are a multiple of BCI (a column tile lies inside one tap) and
// output channel counts that are a multiple of BCO.  Same product as wgrad_kernel, different data path:
//
//  * Pixel rows go to LDS the way they come from memory, [pixel][channel], with 16-byte stores.  The MFMA
//    operands, which need the pixel index contiguous per channel, are read with the transposing LDS load
//    (ds_read_b64_tr_b16): within 16 lanes, lane 4e+c supplies the address of four channels 4c..4c+3 of pixel
//    e, and lane i receives pixels 0..3 of channel i.  Two such loads give the eight pixels per lane of a
//    32x32x16 operand.  No shuffling in registers, no strided LDS stores.
//  * A row's 32-byte blocks are XOR-ed with 2*(pixel % 4): the four pixels x two channel blocks that 32 lanes
//    read together then fall into eight different bank groups.
//  * Gathers are buffer loads as in igemm_ring_kernel (scalar offset = position of the 64-pixel step, lanes on
//    padding or beyond the pixel range get zeros from the bounds check), software-pipelined the same way:
//    step g is multiplied from one LDS stage while step g+1 moves from registers into the other and step g+2
//    is loaded, a few pieces after each group of MFMAs.
//  * The gather origin of a pixel (frame, row, column -> offset and tap validity) is decoded one pixel per
//    thread for NT pixels at a time, a batch ahead of its use.
struct PixInfo {
    uint32_t off;    // byte offset of the pixel's gather origin in the biased x buffer
    uint32_t mask;   // as RowInfo::mask; 0 beyond the block's pixel range
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16x8 lds_read_tr_pair(const unsigned char* p0, const unsigned char* p1) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p1);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int BCO, int BCI, int WM, int WN, bool AFF = false>
__global__ void __launch_bounds__(WM * WN * 64) wgrad_tr_kernel(WgradArgs a) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BCO / WM, TN = BCI / WN;       // wavefront tile
    constexpr int MI = TM / 32, NJ = TN / 32;
    constexpr int PXS = WMK;                          // pixels per step
    // bytes per pixel row of the two operands in LDS
    constexpr int ROWA = BCO * 2, ROWB = BCI * 2;
    constexpr int STAGE = PXS * (ROWA + ROWB);
    constexpr int AVR = BCO / 8, BVR = BCI / 8;       // 16-byte pieces per row
    constexpr int RA = NT / AVR;                      // dy rows per load pass
    constexpr int PA = PXS / RA, PB = PXS * BVR / NT; // pieces per thread and step
    constexpr int NP = PA + PB;
    // x pieces: piece tid + j*NT is vector (tid + j*NT) % BVR of row (tid + j*NT) / BVR.  When NT is a multiple
    // of BVR the vector is the same for all of a thread's pieces and the rows are NT/BVR apart.
    constexpr bool BREG = NT % BVR == 0;
    constexpr int SPB = NT / PXS;                     // steps per decoded batch of NT pixels
    constexpr int KS = PXS / 16;
    static_assert(RA % 4 == 0 && PXS % RA == 0 && (PXS * BVR) % NT == 0, "tile / thread mismatch");
    static_assert(!BREG || (NT / BVR) % 4 == 0, "row swizzle of a thread's pieces must agree");
    static_assert(NT % PXS == 0 && SPB >= 4, "whole steps per batch; a batch is decoded at least three steps ahead");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][STAGE], then the pixel table
    PixInfo* s_pix = (PixInfo*)(smem + 2 * STAGE);                           // [2][NT]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    // One-dimensional grid.  Workgroups go to the eight XCDs round-robin by index, and every tile of D reads the
    // same pixels of a chunk (all of dy for its row tile, all of x for its column tile): with a.group == 8 the
    // tiles of one chunk are the indices 8 apart inside a run of 8 * tiles, so they share an XCD, start together
    // and find each other's rows in that XCD's L2.  a.group == 0 (few chunks): chunk fastest, tile slowest.
    const int bid = (int)blockIdx.x;
    const int tile_id = a.group ? (bid >> 3) % a.tiles : bid / a.nchunks;
    const int chunk_id = a.group ? (bid / (8 * a.tiles)) * 8 + (bid & 7) : bid % a.nchunks;
    const int co0 = (tile_id / a.col_tiles) * BCO;
    const int j0 = (tile_id % a.col_tiles) * BCI;
    const long mbeg = (long)chunk_id * a.chunk;
    long mend = mbeg + a.chunk;
    if (mend > a.M) mend = a.M;
    if (mbeg >= mend) return;
    const int nsteps = (int)((mend - mbeg + PXS - 1) / PXS);
    const int hw = a.Ho * a.Wo;
    const int bias_el = (a.pad * a.W + a.pad) * a.pitch;
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(a.dy, (uint32_t)(a.M * a.Cout * 2));
    const __amdgpu_buffer_rsrc_t rsrc_y = make_rsrc(AFF ? a.ay : a.dy, (uint32_t)(a.M * a.Cout * 2));
    const __amdgpu_buffer_rsrc_t rsrc_b =
        make_rsrc(a.x - bias_el, (uint32_t)(((long)a.F * a.H * a.W * a.pitch + (a.Cin - a.pitch) + bias_el) * 2));

    // ---- this thread's pieces: dy rows arow + i*RA, x rows brow + j*RB of every step
    const int avec = tid % AVR, arow = tid / AVR;
    float ka[8], kb[8], kc[8];                        // AFF: coefficients of this thread's eight output channels
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int c = co0 + avec * 8 + q;
        ka[q] = AFF ? a.aff[c] : 1.f;
        kb[q] = AFF ? a.aff[a.Cout + c] : 0.f;
        kc[q] = AFF ? a.aff[2 * a.Cout + c] : 0.f;
    }
    uint32_t a_off[PA];
#pragma unroll
    for (int i = 0; i < PA; ++i) a_off[i] = (uint32_t)(((arow + i * RA) * a.Cout + co0 + avec * 8) * 2);
    auto swz_a = [](int r) { return ROWA >= 256 ? 2 * (r & 3) : 2 * ((r >> 1) & 1); };
    // (rows of 384 bytes, like rows of 128, start half a bank cycle apart: row parity already separates two of the four
    //  pixels, and an XOR that only touches bit 1 of the block index stays inside the row's twelve blocks)
    auto swz_b = [](int r) { return ROWB % 256 == 0 ? 2 * (r & 3) : 2 * ((r >> 1) & 1); };
    constexpr int PBV = BREG ? 1 : PB;               // distinct (need, const) pairs per thread
    uint32_t b_need[PBV], b_const[PBV];
    int b_row[PB], b_wr[PB];                          // row within the step, LDS position
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        const int p = tid + q * NT;
        const int bvec = BREG ? tid % BVR : p % BVR;
        b_row[q] = BREG ? tid / BVR + q * (NT / BVR) : p / BVR;
        b_wr[q] = PXS * ROWA + b_row[q] * ROWB + ((((bvec >> 1) ^ swz_b(b_row[q])) << 5) | ((bvec & 1) << 4));
        if (q < PBV) {
            const int j = j0 + bvec * 8;             // column of D: (tap, input channel)
            const int tap = j / a.Cin, ci = j - tap * a.Cin;
            const int kw = tap % a.KW, kh = (tap / a.KW) % a.KH, kt = tap / (a.KW * a.KH);
            const int d = kt - a.KT / 2 + group_dt(ci, a.fold);
            b_need[q] = (1u << kh) | (1u << (8 + kw)) | (d > 0 ? 1u << 30 : 0u) | (d < 0 ? 1u << 31 : 0u);
            b_const[q] = (uint32_t)((d * a.H * a.W * a.pitch + (kh * a.W + kw) * a.pitch + ci) * 2);
        }
    }
    // LDS positions of the pieces (row r, 16-byte vector v): 32-byte block (v/2) ^ 2*(r%4), half v%2
    // (rows of 128 bytes hold only four blocks and two of them span the banks: there the XOR is 2*((r/2)%2))
    const int a_wr = arow * ROWA + ((((avec >> 1) ^ swz_a(arow)) << 5) | ((avec & 1) << 4));

    // ---- operand read addresses (see the layout of the transposing load above): lane = 32*kg + 16*mblk + 4*e + c
    int a_rd[MI], b_rd[NJ];
    {
        const int c = lane & 3, e = (lane >> 2) & 3, mblk = (lane >> 4) & 1, kg = lane >> 5;
#pragma unroll
        for (int i = 0; i < MI; ++i)
            a_rd[i] = (8 * kg + e) * ROWA + ((((wm * (TM / 16) + i * 2 + mblk) ^ swz_a(e)) << 5) | (c << 3));
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            b_rd[j] = PXS * ROWA + (8 * kg + e) * ROWB + ((((wn * (TN / 16) + j * 2 + mblk) ^ swz_b(e)) << 5) | (c << 3));
    }

    auto decode = [&](int batch) {   // one pixel per thread
        const long m = mbeg + (long)batch * NT + tid;
        PixInfo info;
        info.off = 0;
        info.mask = 0;
        if (m < mend) {
            const int f = (int)(m / hw);
            const int pix = (int)(m - (long)f * hw);
            const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
            const int ih = oh * a.stride - a.pad, iw = ow * a.stride - a.pad;
            const int t = f % a.T;
            uint32_t mask = 0;
            for (int kh = 0; kh < a.KH; ++kh)
                if (ih + kh >= 0 && ih + kh < a.H) mask |= 1u << kh;
            for (int kw = 0; kw < a.KW; ++kw)
                if (iw + kw >= 0 && iw + kw < a.W) mask |= 1u << (8 + kw);
            if (t + 1 < a.T) mask |= 1u << 30;
            if (t >= 1) mask |= 1u << 31;
            info.off = (uint32_t)((((long)f * a.H * a.W + (long)ih * a.W + iw) * a.pitch + bias_el) * 2);
            info.mask = mask;
        }
        s_pix[(batch & 1) * NT + tid] = info;
    };

    struct Plan {
        uint32_t v[NP];
        int soff_a;
    };
    auto plan = [&](int st) {   // step st (may lie beyond the last one: all zeros then)
        Plan p;
        const long left = mend - (mbeg + (long)st * PXS);        // pixels from the step's first one to the end
        p.soff_a = left > 0 ? (int)((mbeg + (long)st * PXS) * a.Cout * 2) : 0;
#pragma unroll
        for (int i = 0; i < PA; ++i) p.v[i] = (arow + i * RA) < left ? a_off[i] : OOB_OFFSET;
        const PixInfo* tab = s_pix + ((st / SPB) & 1) * NT + (st % SPB) * PXS;
#pragma unroll
        for (int j = 0; j < PB; ++j) {
            const PixInfo pi = tab[b_row[j]];
            const uint32_t need = b_need[BREG ? 0 : j], cst = b_const[BREG ? 0 : j];
            p.v[PA + j] = (left > 0 && (pi.mask & need) == need) ? pi.off + cst : OOB_OFFSET;
        }
        return p;
    };
    u32x4 greg[NP];
    u32x4 gy[AFF ? PA : 1];       // AFF: the BatchNorm input beside each dz piece
    uint32_t gvalid = 0;          // AFF: bit i = piece i lies inside the pixel range (rows beyond it must stay zero)
    auto load_piece = [&](const Plan& p, int i) {
        greg[i] = i < PA ? __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, (int)p.v[i], p.soff_a, 0)
                         : __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, (int)p.v[i], 0, 0);
        if (AFF && i < PA) {
            gy[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_y, (int)p.v[i], p.soff_a, 0);
            gvalid = p.v[i] != OOB_OFFSET ? gvalid | (1u << i) : gvalid & ~(1u << i);
        }
    };
    auto store_piece = [&](int stage, int i) {
        const int pos = i < PA ? a_wr + i * RA * ROWA : b_wr[i < PA ? 0 : i - PA];
        u32x4 v = greg[i];
        if (AFF && i < PA) {
            const u32x4 y = gy[i];
            const bool in = (gvalid >> i) & 1u;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = fmaf(ka[2 * e], __uint_as_float(v[e] << 16), fmaf(kb[2 * e], __uint_as_float(y[e] << 16), kc[2 * e]));
                const float hi = fmaf(ka[2 * e + 1], __uint_as_float(v[e] & 0xffff0000u),
                                      fmaf(kb[2 * e + 1], __uint_as_float(y[e] & 0xffff0000u), kc[2 * e + 1]));
                v[e] = in ? pack_bf16x2(lo, hi) : 0u;
            }
        }
        *(u32x4*)(smem + stage * STAGE + pos) = v;
    };

    f32x16 acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    decode(0);
    __syncthreads();
    {
        const Plan p0 = plan(0);
#pragma unroll
        for (int i = 0; i < NP; ++i) load_piece(p0, i);
#pragma unroll
        for (int i = 0; i < NP; ++i) store_piece(0, i);
        const Plan p1 = plan(1);
#pragma unroll
        for (int i = 0; i < NP; ++i) load_piece(p1, i);
    }
    Plan pl = plan(2);

    for (int st = 0; st < nsteps; ++st) {
        // batch b+1 is decoded during the first step of batch b; it is first read by the plan of its first
        // step, two steps before that step is multiplied
        if (st % SPB == 0 && (st / SPB + 1) * SPB < nsteps) decode(st / SPB + 1);
        __syncthreads();   // stage st % 2 is complete, and everybody is done with the other stage
        const unsigned char* cur = smem + (st & 1) * STAGE;
        constexpr int PPK = (NP + KS - 2) / (KS - 1);
        bf16x8 af[2][MI], bfr[2][NJ];
#pragma unroll
        for (int i = 0; i < MI; ++i) af[0][i] = lds_read_tr_pair(cur + a_rd[i], cur + a_rd[i] + 4 * ROWA);
#pragma unroll
        for (int j = 0; j < NJ; ++j) bfr[0][j] = lds_read_tr_pair(cur + b_rd[j], cur + b_rd[j] + 4 * ROWB);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cb = ks & 1, nb = cb ^ 1;
            if (ks + 1 < KS) {
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    af[nb][i] = lds_read_tr_pair(cur + a_rd[i] + (ks + 1) * 16 * ROWA, cur + a_rd[i] + ((ks + 1) * 16 + 4) * ROWA);
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    bfr[nb][j] = lds_read_tr_pair(cur + b_rd[j] + (ks + 1) * 16 * ROWB, cur + b_rd[j] + ((ks + 1) * 16 + 4) * ROWB);
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cb][i], bfr[cb][j], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int q = ks * PPK; q < (ks + 1) * PPK && q < NP; ++q) {
                store_piece((st & 1) ^ 1, q);
                load_piece(pl, q);
            }
            __builtin_amdgcn_sched_barrier(0);   // keep the pieces where they are
        }
        if (st + 1 < nsteps) pl = plan(st + 3);
    }

    // ---- fp32 atomics: lane = column (input channel), register = row (output channel)
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int col = j0 + wn * TN + j * 32 + (lane & 31);
            const int tap = col / a.Cin, ci = col - tap * a.Cin;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int co = co0 + wm * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                atomicAdd(a.dw + (long)co * a.so + (long)ci * a.si + (long)tap * a.st, acc[i][j][r]);
            }
        }
}

template <int BCO, int BCI, int WM, int WN, bool AFF = false>
static int launch_wgrad_tr(WgradArgs& a, int Cout, int blocks_per_cu, const char* name, hipStream_t s) {
    constexpr int NT = WM * WN * 64;
    a.col_tiles = a.K / BCI;
    const int tiles = (Cout / BCO) * a.col_tiles;
    long want = (long)blocks_per_cu * num_cu() / tiles;
    if (want < 1) want = 1;
    const char* xe = getenv("TSM_WGRAD_XCD");   // TSM_WGRAD_XCD=0 (read at every call): chunk-fastest block order everywhere
    // (whole groups of eight chunks, all blocks resident at once; not where rounding down to a multiple of
    //  eight would idle more than 3 % of the CUs)
    const bool grouped = !(xe && xe[0] == '0') && tiles > 1 && want >= 16 && (want & 7) * 100 <= want * 3;
    if (grouped) want = want / 8 * 8;
    long chunk = (a.M + want - 1) / want;
    // at least 16 K steps per block: below that the fp32 atomics of the tile (one per block) outweigh the
    // parallelism gained (measured at 64 frames: 1x1 layers of the last three stages 10 % faster)
    if (chunk < 16L * WMK) chunk = 16L * WMK;
    a.chunk = (chunk + WMK - 1) / WMK * WMK;
    a.tiles = tiles;
    a.nchunks = (int)((a.M + a.chunk - 1) / a.chunk);
    a.group = grouped ? 8 : 0;
    const dim3 grid((unsigned)((grouped ? (a.nchunks + 7) / 8 * 8 : a.nchunks) * tiles));
    auto kern = wgrad_tr_kernel<BCO, BCI, WM, WN, AFF>;
    const size_t smem = (size_t)2 * WMK * (BCO * 2 + BCI * 2) + (size_t)2 * NT * sizeof(PixInfo);
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "wgrad: cannot raise dynamic LDS limit");
        configured = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(NT), smem, s, a);
    return check_launch(name);
}

bool conv_mfma_wgrad_affine_ok(const ConvP& p) {
    const long limit = 0x7ff00000L;
    const int pitch = p.pix_pitch();
    return p.rows_out() * p.Cout * 2 < limit && (p.rows_in() * (long)pitch + p.Cin + (long)(p.pad * p.W + p.pad) * pitch) * 2 < limit &&
           p.Cin % 64 == 0 && p.Cout == 64 && p.K() % 256 == 0 && pitch != p.Cin;
}

int conv_mfma_wgrad(const ConvP& p, const bf16_t* x, const bf16_t* dy, float* dw, int cin_real, bool packed,
                    hipStream_t s, const bf16_t* affine_y, const float* affine_coef) {
    WgradArgs a;
    a.x = x; a.dy = dy; a.dw = dw; a.cin_real = cin_real;
    a.ay = affine_y; a.aff = affine_coef;
    if ((affine_y != nullptr) != (affine_coef != nullptr)) return fail(TSM_ERR_NULLPTR, "wgrad: the affine form needs both its operands");
    if (affine_y && !(conv_mfma_wgrad_affine_ok(p) && cin_real == p.Cin))
        return fail(TSM_ERR_UNSUPPORTED, "wgrad: this layer's kernel cannot form dy while loading");
    if (packed) {   // [Cout][taps][p.Cin]: consecutive lanes (channels) hit consecutive addresses
        a.so = (long)p.taps() * p.Cin; a.si = 1; a.st = p.Cin;
    } else {        // ABI order [Cout][cin_real][taps]
        a.so = (long)cin_real * p.taps(); a.si = p.taps(); a.st = 1;
    }
    a.F = p.F; a.T = p.T; a.H = p.H; a.W = p.W; a.Cin = p.Cin; a.pitch = p.pix_pitch();
    a.Ho = p.Ho; a.Wo = p.Wo; a.Cout = p.Cout;
    a.KT = p.KT; a.KH = p.KH; a.KW = p.KW; a.stride = p.stride; a.pad = p.pad;
    a.fold = p.fold;
    a.M = p.rows_out();
    a.K = (int)p.K();
    if (a.M == 0) return TSM_OK;
    {   // transposing-read kernels: channel counts that fill whole tiles, tensors below 2 GiB
        static int enabled = -1;   // TSM_WGRAD_TR=0 keeps the register-transposing kernels everywhere (for comparisons)
        if (enabled < 0) {
            const char* e = getenv("TSM_WGRAD_TR");
            enabled = (e && e[0] == '0') ? 0 : 1;
        }
        const long limit = 0x7ff00000L;
        const bool fits = a.M * p.Cout * 2 < limit &&
                          (p.rows_in() * (long)a.pitch + p.Cin + (long)(p.pad * p.W + p.pad) * a.pitch) * 2 < limit;
        // (a pixel pitch other than the channel count -- the stem in space-to-depth form -- only runs here)
        if ((enabled || a.pitch != p.Cin) && fits && cin_real == p.Cin && p.Cin % 64 == 0 && p.Cout % 64 == 0) {
            // blocks per CU follow from the LDS footprint of two stages
            if (p.Cout % 256 == 0 && p.Cin % 128 == 0) return launch_wgrad_tr<256, 128, 4, 2>(a, p.Cout, 1, "wgrad_tr_256x128", s);
            if (p.Cout % 256 == 0) return launch_wgrad_tr<256, 64, 4, 1>(a, p.Cout, 1, "wgrad_tr_256x64", s);
            if (p.Cout % 128 == 0 && p.Cin % 128 == 0) return launch_wgrad_tr<128, 128, 2, 2>(a, p.Cout, 2, "wgrad_tr_128x128", s);
            // (a column tile may span several taps: 64 input channels x 4 taps fill the 256 columns too)
            if (affine_y) return launch_wgrad_tr<64, 256, 1, 4, true>(a, p.Cout, 1, "wgrad_tr_64x256", s);
            if (a.K % 256 == 0 && (p.Cin % 256 == 0 || a.pitch != p.Cin)) return launch_wgrad_tr<64, 256, 1, 4>(a, p.Cout, 1, "wgrad_tr_64x256", s);
            if (p.taps() == 1) return launch_wgrad_tr<64, 64, 2, 2>(a, p.Cout, 4, "wgrad_tr_64x64", s);
            // 64 input channels and several taps: a column tile of three taps shares the dy tile among them
            // (two blocks per CU: the layer is bound by the latency of its gathers, not by a unit)
            if (a.K % 192 == 0) return launch_wgrad_tr<64, 192, 2, 2>(a, p.Cout, 2, "wgrad_tr_64x192", s);
        }
    }
    if (affine_y) return fail(TSM_ERR_UNSUPPORTED, "wgrad: the affine form needs the transposing-read kernels");
    if (a.pitch != p.Cin) return fail(TSM_ERR_UNSUPPORTED, "wgrad: a pixel pitch other than the channel count needs the transposing-read kernels");
    // tiles: 128x128 for wide outputs; for <= 64 output channels a 64x192 tile when K is long enough (the
    // transposed dy tile is then shared by three times as many columns); 64x64 otherwise
    const bool big = p.Cout > 64 && a.K > 64;
    const bool wide = !big && p.Cout <= 64 && a.K >= 192 && a.K % 192 == 0;
    const int bco = big ? 128 : 64, bci = big ? 128 : (wide ? 192 : 64);
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
    else if (wide)
        wgrad_kernel<64, 192><<<grid, dim3(256), 0, s>>>(a);
    else
        wgrad_kernel<64, 64><<<grid, dim3(256), 0, s>>>(a);
    return check_launch(big ? "wgrad_128x128" : (wide ? "wgrad_64x192" : "wgrad_64x64"));
}

// ---- 3x3 + 1x1 in one kernel (inference) ------------------------------------------------------------------------
bool conv_mfma_fused_tail_supported(const ConvP& p2, const ConvP& p3) {
    const char* e = getenv("TSM_FUSED_TAIL");   // TSM_FUSED_TAIL=0 keeps one kernel per convolution (read at every call)
    if (e && e[0] == '0') return false;
    const int mid = p2.Cin;
    if (!(mid == 64 || mid == 128)) return false;
    if (p2.Cout != mid || p3.Cin != mid || p3.Cout != 4 * mid) return false;
    if (p2.KT != 1 || p2.KH != 3 || p2.KW != 3 || p2.pad != 1 || p2.fold != 0 || p2.pitch != 0 || p2.stride < 1 || p2.stride > 2) return false;
    if (p3.KT != 1 || p3.KH != 1 || p3.KW != 1 || p3.pad != 0 || p3.stride != 1 || p3.fold != 0 || p3.pitch != 0) return false;
    if (p3.H != p2.Ho || p3.W != p2.Wo || p3.F != p2.F) return false;
    const long limit = 0x7ff00000L;
    if ((p2.rows_in() + p2.W + 1) * (long)mid * 2 >= limit || p3.rows_out() * 4L * mid * 2 >= limit) return false;
    // fewer than three quarters of a round of tiles: the two-kernel path spreads such layers over more blocks
    // (TSM_FUSED_TAIL_MIN_TILES=<n>, read at every call, moves the threshold: tests and comparisons set it)
    const char* t = getenv("TSM_FUSED_TAIL_MIN_TILES");
    const long min_tiles = t ? atol(t) : ((long)num_cu() * 3 + 3) / 4;
    if ((p2.rows_out() + 255) / 256 < min_tiles) return false;
    return true;
}

template <int MID, bool STREAM>
static int launch_fused_tail(const TailArgs& a, long rows, hipStream_t s) {
    auto kern = fused_tail_kernel<MID, STREAM>;
    constexpr size_t smem = (size_t)2 * (256 + 128) * BK * sizeof(bf16_t) + (size_t)128 * (128 + 8) * sizeof(bf16_t) +
                            (size_t)256 * sizeof(RowInfo) + (size_t)10 * MID * sizeof(float);
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return fail(TSM_ERR_LAUNCH, "fused_tail: cannot raise dynamic LDS limit");
        configured = true;
    }
    const int grid = igemm_grid((int)((rows + 255) / 256), 64, 64, 1);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, s, a);
    return check_launch(MID == 64 ? "fused_tail_64" : "fused_tail_128");
}

int conv_mfma_fused_tail(const ConvP& p2, const ConvP& p3, const bf16_t* x, const bf16_t* w2p, const bf16_t* w3p,
                         const float* sc2, const float* sh2, const float* sc3, const float* sh3, const bf16_t* res,
                         bf16_t* out, hipStream_t s) {
    if (!conv_mfma_fused_tail_supported(p2, p3)) return fail(TSM_ERR_UNSUPPORTED, "fused tail: no kernel for this pair of layers");
    if (!res) return fail(TSM_ERR_NULLPTR, "fused tail: the shortcut is required");
    TailArgs a;
    a.src = x; a.w2 = w2p; a.w3 = w3p; a.sc2 = sc2; a.sh2 = sh2; a.sc3 = sc3; a.sh3 = sh3; a.res = res; a.dst = out;
    a.F = p2.F; a.Hs = p2.H; a.Ws = p2.W; a.Hd = p2.Ho; a.Wd = p2.Wo; a.stride = p2.stride;
    const long rows = p2.rows_out();
    if (rows == 0) return TSM_OK;
    const bool stream = rows * 4L * p2.Cin * 2 > (64L << 20);
    if (p2.Cin == 64) return stream ? launch_fused_tail<64, true>(a, rows, s) : launch_fused_tail<64, false>(a, rows, s);
    return stream ? launch_fused_tail<128, true>(a, rows, s) : launch_fused_tail<128, false>(a, rows, s);
}

}  // namespace tsm
