// Stand-alone temporal shift S(x) / S^T(g) (paper section 2, Fig. 1) and the
// NTCHW <-> NTHWC frame transposes used by the compatibility paths.
//
// The shift has no arithmetic: every kernel here is a gather copy whose only
// cost is one read and one write of the tensor, so the design goal is plain
// 16-byte coalesced traffic at HBM rate.
#include <stdarg.h>
#include <string.h>
#include <map>
#include <string>
#include <vector>
#include "common.h"
#include "internal.h"

namespace tsm {

// ---- error plumbing ---------------------------------------------------------
static thread_local char g_err[512] = "no error";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// ---- optional per-launch timing (measurement aid) ----------------------------------
// While enabled, a HIP event is recorded on the profiled stream after every kernel
// launch that goes through check_launch(); the time between consecutive events is
// booked on the kernel class named by `what`.
struct ProfState {
    bool on = false;
    hipStream_t stream = nullptr;
    std::vector<hipEvent_t> pool;
    std::vector<const char*> names;   // names[i] belongs to event i+1 (event 0 is the start mark)
    size_t used = 0;
};
static thread_local ProfState g_prof;

static hipEvent_t prof_next_event() {
    if (g_prof.used == g_prof.pool.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        g_prof.pool.push_back(e);
    }
    return g_prof.pool[g_prof.used++];
}

bool profiling_active() { return g_prof.on; }

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TSM_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
    if (g_prof.on) {
        hipEvent_t ev = prof_next_event();
        if (ev && hipEventRecord(ev, g_prof.stream) == hipSuccess) g_prof.names.push_back(what);
    }
    return TSM_OK;
}

// ---- channels-innermost shift ------------------------------------------------
// One thread moves one V-sized piece of one pixel's channel vector.  `dir` is +1 for S (group 1 reads t+1,
// group 2 reads t-1) and -1 for S^T.  foldv/cv: fold and C measured in V units.
// blockIdx.y walks the frames (frame index and clip position are uniform in a block), blockIdx.x and the thread
// cover the frame's vectors: 32-bit index arithmetic, no division by the frame size per thread.  Measured on a
// [64,8,256,56,56] bf16 tensor: one vector per thread beats two or four (5.3 TB/s), blocks of 128 threads beat
// 256 and 1024 (6.33 / 6.28 / 6.0 TB/s), regular loads with nontemporal stores beat nontemporal loads (5.9 TB/s).
// A second sweep with all loads of a thread issued before its stores: 2 / 4 vectors per thread 6.1-6.2 / 5.7-6.0 TB/s,
// grid-stride blocks of 256 threads with 4 or 8 vectors 5.5 / 5.2, blocks of 64 / 192 / 256 threads 6.33 / 6.08 / 6.24,
// regular stores 6.3, frames on the fast grid axis 5.1 -- against 6.27-6.39 for this form (the memory system here
// prefers many small independent wavefronts; the figure itself drifts by 1-2 % within a process).
static constexpr int SHIFT_U = 1;     // vectors per thread
static constexpr int SHIFT_NT = 128;  // threads per block
template <typename V>
__global__ void __launch_bounds__(SHIFT_NT) shift_nthwc_kernel(const V* __restrict__ x, V* __restrict__ y,
                                                               unsigned frames, int T, unsigned frame_v,
                                                               unsigned cv, unsigned foldv, int dir) {
    for (unsigned f = blockIdx.y; f < frames; f += gridDim.y) {
        const int t = (int)(f % (unsigned)T);
        const V* xf = x + (size_t)f * frame_v;
        V* yf = y + (size_t)f * frame_v;
        const bool up_ok = t + dir >= 0 && t + dir < T;        // group 1 reads frame t + dir
        const bool dn_ok = t - dir >= 0 && t - dir < T;        // group 2 reads frame t - dir
        const ptrdiff_t up = (ptrdiff_t)dir * (ptrdiff_t)frame_v;
#pragma unroll
        for (int u = 0; u < SHIFT_U; ++u) {
            const unsigned j = (blockIdx.x * SHIFT_U + u) * (unsigned)SHIFT_NT + threadIdx.x;
            if (j >= frame_v) break;
            const unsigned c = j % cv;
            // one load site for all three channel groups (lanes of a wavefront fall into all of them)
            const bool g1 = c < foldv, g2 = !g1 && c < 2 * foldv;
            const ptrdiff_t off = g1 ? up : (g2 ? -up : 0);
            const bool valid = g1 ? up_ok : (g2 ? dn_ok : true);
            V v = V{};
            if (valid) v = xf[j + off];
            __builtin_nontemporal_store(v, yf + j);
        }
    }
}

// ---- channel-planes shift (the paper's memory order) ---------------------------
// A (n,t,c) plane of H*W elements is contiguous; it is copied whole from frame
// t+dt or zero-filled.  plane_v = plane size in V units.
template <typename V>
__global__ void __launch_bounds__(256) shift_ntchw_kernel(const V* __restrict__ x, V* __restrict__ y,
                                                          size_t total, int T, int C, int plane_v,
                                                          int fold, int dir) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const size_t plane = i / plane_v;
    const int c = (int)(plane % C);
    const int t = (int)((plane / C) % T);
    int dt = 0;
    if (c < fold) dt = dir;
    else if (c < 2 * fold) dt = -dir;
    const int ts = t + dt;
    V v;
    if (ts >= 0 && ts < T) {
        v = __builtin_nontemporal_load(x + (ptrdiff_t)i + (ptrdiff_t)dt * (ptrdiff_t)C * plane_v);
    } else {
        v = V{};
    }
    __builtin_nontemporal_store(v, y + i);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V>
static int launch_nthwc(const void* x, void* y, size_t bytes, int T, size_t frame_bytes, int c_bytes,
                        int fold_bytes, int dir, hipStream_t s) {
    size_t total = bytes / sizeof(V);
    if (total == 0) return TSM_OK;
    const size_t frame_v = frame_bytes / sizeof(V);
    const size_t frames = total / frame_v;
    if (frame_v > 0x7fffffffull || frames > 0x7fffffffull) return fail(TSM_ERR_SHAPE, "shift: tensor too large");
    const unsigned gx = (unsigned)((frame_v + SHIFT_NT * SHIFT_U - 1) / (SHIFT_NT * SHIFT_U));
    const unsigned gy = (unsigned)(frames < 65535 ? frames : 65535);
    shift_nthwc_kernel<V><<<dim3(gx, gy), dim3(SHIFT_NT), 0, s>>>(
        (const V*)x, (V*)y, (unsigned)frames, T, (unsigned)frame_v, (unsigned)(c_bytes / (int)sizeof(V)),
        (unsigned)(fold_bytes / (int)sizeof(V)), dir);
    return check_launch("shift_nthwc");
}

template <typename V>
static int launch_ntchw(const void* x, void* y, size_t bytes, int T, int C, size_t plane_bytes, int fold,
                        int dir, hipStream_t s) {
    size_t total = bytes / sizeof(V);
    if (total == 0) return TSM_OK;
    size_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffull) return fail(TSM_ERR_SHAPE, "shift: tensor too large");
    shift_ntchw_kernel<V><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
        (const V*)x, (V*)y, total, T, C, (int)(plane_bytes / sizeof(V)), fold, dir);
    return check_launch("shift_ntchw");
}

// dir = +1: S, dir = -1: S^T.  Arguments are validated by the caller.
int shift_launch(const void* x, void* y, int N, int T, int C, int H, int W, int fold, int es, int layout,
                 int dir, hipStream_t s) {
    const size_t bytes = (size_t)N * T * C * H * W * es;
    if (layout == TSM_NTHWC) {
        const int cb = C * es, fb = fold * es;
        const size_t frame = (size_t)H * W * cb;
        if (cb % 16 == 0 && fb % 16 == 0) return launch_nthwc<u32x4>(x, y, bytes, T, frame, cb, fb, dir, s);
        if (cb % 8 == 0 && fb % 8 == 0) return launch_nthwc<u32x2>(x, y, bytes, T, frame, cb, fb, dir, s);
        if (cb % 4 == 0 && fb % 4 == 0) return launch_nthwc<uint32_t>(x, y, bytes, T, frame, cb, fb, dir, s);
        return launch_nthwc<uint16_t>(x, y, bytes, T, frame, cb, fb, dir, s);
    }
    const size_t pb = (size_t)H * W * es;
    if (pb % 16 == 0) return launch_ntchw<u32x4>(x, y, bytes, T, C, pb, fold, dir, s);
    if (pb % 8 == 0) return launch_ntchw<u32x2>(x, y, bytes, T, C, pb, fold, dir, s);
    if (pb % 4 == 0) return launch_ntchw<uint32_t>(x, y, bytes, T, C, pb, fold, dir, s);
    return launch_ntchw<uint16_t>(x, y, bytes, T, C, pb, fold, dir, s);
}

// ---- frame transposes [F][C][P] <-> [F][P][C] -----------------------------------
// 32x32 element tiles through LDS; E is a 2- or 4-byte unsigned type.
template <typename E>
__global__ void __launch_bounds__(256) transpose_kernel(const E* __restrict__ in, E* __restrict__ out,
                                                        int rows, int cols) {
    // in: [F][rows][cols] -> out: [F][cols][rows]
    __shared__ E tile[32][33];
    const size_t fo = (size_t)blockIdx.z * rows * cols;
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int j = ty; j < 32; j += 8) {
        int r = r0 + j, c = c0 + tx;
        if (r < rows && c < cols) tile[j][tx] = in[fo + (size_t)r * cols + c];
    }
    __syncthreads();
    for (int j = ty; j < 32; j += 8) {
        int c = c0 + j, r = r0 + tx;
        if (r < rows && c < cols) out[fo + (size_t)c * rows + r] = tile[tx][j];
    }
}

// Transposes F frames of [rows][cols] elements of size es into [cols][rows].
int transpose_frames(const void* in, void* out, int F, int rows, int cols, int es, hipStream_t s) {
    if (F <= 0 || rows <= 0 || cols <= 0) return TSM_OK;
    dim3 grid(cdiv(cols, 32), cdiv(rows, 32), F);
    if (es == 2)
        transpose_kernel<uint16_t><<<grid, dim3(256), 0, s>>>((const uint16_t*)in, (uint16_t*)out, rows, cols);
    else
        transpose_kernel<uint32_t><<<grid, dim3(256), 0, s>>>((const uint32_t*)in, (uint32_t*)out, rows, cols);
    return check_launch("transpose_frames");
}

static int shift_entry(const void* x, void* y, int N, int T, int C, int H, int W, int fold_div, int dtype,
                       int layout, void* stream, int dir) {
    if (!x || !y) return fail(TSM_ERR_NULLPTR, "tsm_shift: null tensor pointer");
    if (N <= 0 || T <= 0 || C <= 0 || H <= 0 || W <= 0)
        return fail(TSM_ERR_SHAPE, "tsm_shift: non-positive dimension N=%d T=%d C=%d H=%d W=%d", N, T, C, H, W);
    if (dtype != TSM_F32 && dtype != TSM_BF16) return fail(TSM_ERR_DTYPE, "tsm_shift: unknown dtype %d", dtype);
    if (layout != TSM_NTCHW && layout != TSM_NTHWC) return fail(TSM_ERR_LAYOUT, "tsm_shift: unknown layout %d", layout);
    int fold = 0;
    if (fold_of(C, fold_div, &fold) != TSM_OK) return fail(TSM_ERR_FOLD, "tsm_shift: invalid fold_div %d for C=%d", fold_div, C);
    if (!aligned16(x) || !aligned16(y)) return fail(TSM_ERR_ALIGN, "tsm_shift: pointers must be 16-byte aligned");
    const size_t bytes = (size_t)N * T * C * H * W * dtype_size(dtype);
    const char* xb = (const char*)x;
    const char* yb = (const char*)y;
    if (xb < yb + bytes && yb < xb + bytes) return fail(TSM_ERR_SHAPE, "tsm_shift: x and y overlap");
    return shift_launch(x, y, N, T, C, H, W, fold, (int)dtype_size(dtype), layout, dir, (hipStream_t)stream);
}

}  // namespace tsm

extern "C" {

const char* tsm_last_error(void) { return tsm::g_err; }

int tsm_profile_begin(void* stream) {
    using namespace tsm;
    g_prof.used = 0;
    g_prof.names.clear();
    g_prof.stream = (hipStream_t)stream;
    hipEvent_t ev = prof_next_event();
    if (!ev || hipEventRecord(ev, g_prof.stream) != hipSuccess) return fail(TSM_ERR_LAUNCH, "tsm_profile_begin: cannot record event");
    g_prof.on = true;
    return TSM_OK;
}

int tsm_profile_end(char* report, size_t report_cap) {
    using namespace tsm;
    if (!g_prof.on) return fail(TSM_ERR_UNSUPPORTED, "tsm_profile_end: profiling was not started");
    g_prof.on = false;
    if (!report || report_cap == 0) return fail(TSM_ERR_NULLPTR, "tsm_profile_end: null report buffer");
    if (hipStreamSynchronize(g_prof.stream) != hipSuccess) return fail(TSM_ERR_LAUNCH, "tsm_profile_end: synchronise failed");
    std::map<std::string, std::pair<long, double>> agg;
    for (size_t i = 0; i < g_prof.names.size(); ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.pool[i], g_prof.pool[i + 1]) != hipSuccess) continue;
        auto& a = agg[g_prof.names[i]];
        a.first += 1;
        a.second += ms;
    }
    size_t off = 0;
    report[0] = 0;
    for (auto& kv : agg) {
        int n = snprintf(report + off, report_cap - off, "%s %ld %.6f\n", kv.first.c_str(), kv.second.first, kv.second.second);
        if (n < 0 || (size_t)n >= report_cap - off) break;
        off += (size_t)n;
    }
    return TSM_OK;
}

int tsm_shift_fwd(const void* x, void* y, int N, int T, int C, int H, int W, int fold_div, int dtype, int layout,
                  void* stream) {
    return tsm::shift_entry(x, y, N, T, C, H, W, fold_div, dtype, layout, stream, +1);
}

int tsm_shift_bwd(const void* gy, void* gx, int N, int T, int C, int H, int W, int fold_div, int dtype, int layout,
                  void* stream) {
    return tsm::shift_entry(gy, gx, N, T, C, H, W, fold_div, dtype, layout, stream, -1);
}

}  // extern "C"
