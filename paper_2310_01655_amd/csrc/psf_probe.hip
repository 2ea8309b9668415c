// Measurement aid of libpsf: a pure MFMA loop, so that a benchmark can print what this GPU's
// matrix cores sustain under load next to what the attention kernels reach.  Not part of the
// attention path.
#include "psf_internal.h"

namespace psf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Every wave issues iters x 8 independent v_mfma_f32_32x32x16_bf16 (eight accumulators, so the
// loop is bound by the matrix pipe, not by the dependency between accumulations).  Operands are
// pseudo-random non-zero values derived from the thread index: the power drawn, and with it the
// clock the chip settles at, depends on the data toggling.
__global__ __launch_bounds__(256, 2) void k_probe_mfma(float *__restrict__ sink, int iters)
{
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const unsigned ha = (t * 2654435761u + e * 40503u) >> 9, hb = (t * 2246822519u + e * 9973u) >> 9;
        a[e] = (__bf16)(((int)(ha & 1023) - 512) * (1.0f / 512.0f));
        b[e] = (__bf16)(((int)(hb & 1023) - 512) * (1.0f / 512.0f));
    }
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = f32x16{0};
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink[t] = s;
}

}  // namespace
}  // namespace psf

extern "C" psf_status psf_probe_mfma_loop(int32_t workgroups, int32_t iters, void *sink, void *hip_stream)
{
    if (!sink) return PSF_ERR_NULL;
    if (workgroups <= 0 || iters <= 0 || workgroups > 65535) return PSF_ERR_SHAPE;
    hipLaunchKernelGGL(psf::k_probe_mfma, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream,
                       (float *)sink, (int)iters);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}
