// bf16 MFMA path of libpsf (placeholder until the kernels land).
#include "psf_internal.h"
namespace psf {
size_t mfma_workspace_bytes(const Problem &) { return 0; }
psf_status mfma_sketch(const Problem &, const void *, const void *, void *, void *, hipStream_t) { return PSF_ERR_UNSUPPORTED; }
psf_status mfma_attn(const Problem &, const void *, const void *, const void *, const void *, void *, void *, hipStream_t, StageTimer *) { return PSF_ERR_UNSUPPORTED; }
}
