// Measurement aid: what the matrix cores of this chip sustain when nothing else is in the way -- a kernel of
// register-only bf16 MFMAs (no memory, no LDS), so that a figure quoted against the published peak can also be
// read against the achievable one.
#include "internal.h"

namespace tsm {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));

static constexpr int PROBE_CHAINS = 4;           // independent accumulators per wavefront
static constexpr int PROBE_WAVES = 4;            // wavefronts per block, two blocks per CU
static constexpr int PROBE_BLOCKS_PER_CU = 2;

__global__ void __launch_bounds__(PROBE_WAVES * 64, PROBE_BLOCKS_PER_CU) mfma_probe_kernel(int iters, float* sink) {
    probe_f32x16 acc[PROBE_CHAINS];
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    probe_bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
        b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < PROBE_CHAINS; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float v = 0.f;
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) v += acc[c][r];
    if (v == -1.f) sink[0] = v;   // never true (all sums are non-negative); keeps the chain alive
}

}  // namespace tsm

extern "C" int tsm_mfma_probe(int iters, float* sink, double* flops_out, void* stream) {
    using namespace tsm;
    if (iters <= 0 || iters > (1 << 24)) return fail(TSM_ERR_SHAPE, "tsm_mfma_probe: iters out of range");
    if (!sink || !flops_out) return fail(TSM_ERR_NULLPTR, "tsm_mfma_probe: null pointer");
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return fail(TSM_ERR_LAUNCH, "tsm_mfma_probe: cannot query the device");
    const int blocks = cus * PROBE_BLOCKS_PER_CU;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(PROBE_WAVES * 64), 0, (hipStream_t)stream, iters, sink);
    TSM_TRY(check_launch("mfma_probe"));
    *flops_out = (double)blocks * PROBE_WAVES * (double)iters * PROBE_CHAINS * (2.0 * 32 * 32 * 16);
    return TSM_OK;
}
