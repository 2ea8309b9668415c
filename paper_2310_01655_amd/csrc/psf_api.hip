// libpsf entry points: descriptor validation, path selection, workspace sizing, dispatch.
// The operations themselves are defined in include/psf.h (with their citations of
// PolySketchFormer, arXiv 2310.01655); nothing here computes.
#include <initializer_list>
#include <mutex>
#include "psf_internal.h"

namespace psf {

psf_status make_problem(const psf_desc *desc, Problem *out)
{
    if (!desc) return PSF_ERR_NULL;
    if (desc->batch <= 0 || desc->heads <= 0 || desc->n <= 0 || desc->d <= 0 || desc->dv <= 0 ||
        desc->b <= 0)
        return PSF_ERR_SHAPE;
    if (desc->n % desc->b != 0) return PSF_ERR_SHAPE;        // t = n/b blocks (Section 3.1)
    if (desc->p != 2 && desc->p != 4 && desc->p != 8 && desc->p != 16) return PSF_ERR_UNSUPPORTED;
    if (desc->dtype != PSF_F32 && desc->dtype != PSF_BF16) return PSF_ERR_UNSUPPORTED;
    if (desc->feat != PSF_FEAT_SKETCH && desc->feat != PSF_FEAT_EXACT) return PSF_ERR_UNSUPPORTED;
    if (desc->local != PSF_LOCAL_EXACT && desc->local != PSF_LOCAL_SKETCH) return PSF_ERR_UNSUPPORTED;
    if (desc->learned != 0 && desc->learned != 1) return PSF_ERR_UNSUPPORTED;
    if (desc->learned && (desc->feat != PSF_FEAT_SKETCH || desc->p > 8)) return PSF_ERR_UNSUPPORTED;
    const bool needs_r = desc->feat == PSF_FEAT_SKETCH && desc->p > 2;
    if (needs_r && desc->r <= 0) return PSF_ERR_SHAPE;
    if (desc->d > PSF_MAX_DIM || desc->dv > PSF_MAX_DIM || (needs_r && desc->r > PSF_MAX_DIM))
        return PSF_ERR_UNSUPPORTED;
    // units and blocks index grid dimensions y/z (limit 65535); n stays well inside 32 bits
    if ((long long)desc->batch * desc->heads > 65535 || desc->n > (1 << 24) ||
        desc->n / desc->b > 65535)
        return PSF_ERR_UNSUPPORTED;

    Problem pb;
    pb.batch = desc->batch; pb.heads = desc->heads; pb.units = desc->batch * desc->heads;
    pb.n = desc->n; pb.d = desc->d; pb.dv = desc->dv; pb.p = desc->p;
    pb.r = needs_r ? desc->r : desc->d;
    pb.b = desc->b; pb.t = desc->n / desc->b;
    pb.bf16 = desc->dtype == PSF_BF16;
    pb.exact_feat = desc->feat == PSF_FEAT_EXACT;
    pb.local_exact = pb.exact_feat || desc->local == PSF_LOCAL_EXACT;
    pb.per_head = desc->sketch_per_head != 0;
    pb.mcols = (desc->p == 2) ? desc->d : pb.r;
    if (pb.exact_feat) {
        long long F = 1;
        for (int e = 0; e < desc->p; ++e) {
            F *= desc->d;
            if (F > PSF_MAX_FEATURES) return PSF_ERR_UNSUPPORTED;
        }
        pb.F = F;
    } else {
        pb.F = (long long)pb.mcols * pb.mcols;
        if (pb.F > PSF_MAX_FEATURES) return PSF_ERR_UNSUPPORTED;
    }
    // p = 2 is the base case m(x) = x of both algorithms: no network is applied, so a request
    // for learned sketches of that degree is the plain one
    pb.learned = desc->learned != 0 && desc->p > 2;
    pb.g_len = (pb.exact_feat || desc->p == 2) ? 0
               : pb.learned ? psf_learned_len(desc->d, pb.r, desc->p) : psf_g_len(desc->d, pb.r, desc->p);
    *out = pb;
    return PSF_OK;
}

int select_path(const Problem &pb)
{
    const bool shapes = (pb.r == 32 || pb.r == 64) && pb.d == pb.dv && (pb.d == 64 || pb.d == 128) &&
                        (pb.p == 4 || pb.p == 8) && pb.b % 256 == 0;
    // learned sketches included; the in-block rule of Section 3.1 (weights from the sketches) with
    // Gaussian sketches, except d = 128 with r = 32 (a key tile of m(K) rows is half a copy there)
    const bool local_ok = pb.local_exact || (!pb.learned && !(pb.d == 128 && pb.r == 32));
    // p = 2 (m(x) = x, the sketch size is d): d = dv = 64, either in-block rule (they coincide)
    const bool base_case = pb.p == 2 && pb.d == 64 && pb.dv == 64 && pb.b % 256 == 0;
    return (pb.bf16 && !pb.exact_feat && ((local_ok && shapes) || base_case)) ? 1 : 0;
}

psf_status StageTimer::begin(hipStream_t s)
{
    on = false; stream = s; count = 0;
    for (int i = 0; i <= kMax; ++i) {
        if (hipEventCreate(&ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);   // nothing is left behind
            return PSF_ERR_HIP;
        }
    }
    if (hipEventRecord(ev[0], stream) != hipSuccess) {
        for (int j = 0; j <= kMax; ++j) (void)hipEventDestroy(ev[j]);
        return PSF_ERR_HIP;
    }
    on = true;
    return PSF_OK;
}

void StageTimer::mark()
{
    if (!on || count >= kMax) return;
    ++count;
    (void)hipEventRecord(ev[count], stream);
}

psf_status StageTimer::finish(float *ms, int cap, int *written)
{
    psf_status st = PSF_OK;
    if (hipStreamSynchronize(stream) != hipSuccess) st = PSF_ERR_HIP;
    int w = 0;
    for (int i = 0; i < count && i < cap && st == PSF_OK; ++i) {
        if (hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]) != hipSuccess) st = PSF_ERR_HIP;
        ++w;
    }
    for (int i = 0; i <= kMax; ++i) (void)hipEventDestroy(ev[i]);
    if (written) *written = w;
    on = false;
    return st;
}

// The bf16 MFMA kernels read and write the caller's tensors in 16-byte pieces.
static bool aligned16(std::initializer_list<const void *> tensors)
{
    for (const void *p : tensors)
        if (((uintptr_t)p & 15u) != 0) return false;
    return true;
}

static psf_status run_attn(const psf_desc *desc, const void *Q, const void *K, const void *V,
                           const void *G, void *O, void *ws, size_t ws_bytes, void *stream,
                           StageTimer *tm)
{
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    if (!Q || !K || !V || !O) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    const size_t need = psf_workspace_bytes(desc);
    if (need > 0 && !ws) return PSF_ERR_NULL;
    if (ws_bytes < need) return PSF_ERR_WORKSPACE;
    if (((uintptr_t)ws & 255u) != 0) return PSF_ERR_WORKSPACE;
    if (select_path(pb) == 1 && !aligned16({Q, K, V, G, O})) return PSF_ERR_ALIGNMENT;
    hipStream_t s = (hipStream_t)stream;
    return select_path(pb) == 1 ? mfma_attn(pb, Q, K, V, G, O, ws, s, tm)
                                : general_attn(pb, Q, K, V, G, O, ws, s, tm);
}

static psf_status run_noncausal(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                const void *G, void *O, void *ws, size_t ws_bytes, void *stream, StageTimer *tm)
{
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    if (!Q || !K || !V || !O) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    const size_t need = psf_noncausal_workspace_bytes(desc);
    if (need > 0 && !ws) return PSF_ERR_NULL;
    if (ws_bytes < need) return PSF_ERR_WORKSPACE;
    if (((uintptr_t)ws & 255u) != 0) return PSF_ERR_WORKSPACE;
    if (select_path(pb) == 1 && !aligned16({Q, K, V, G, O})) return PSF_ERR_ALIGNMENT;
    hipStream_t s = (hipStream_t)stream;
    return select_path(pb) == 1 ? mfma_attn_noncausal(pb, Q, K, V, G, O, ws, s, tm)
                                : general_attn(pb, Q, K, V, G, O, ws, s, tm, true);
}

// The backward pass runs on MFMA for the shapes of the bf16 forward path it covers.
static bool bwd_on_mfma(const Problem &pb) { return select_path(pb) == 1 && mfma_bwd_supported(pb); }

static psf_status run_bwd(const psf_desc *desc, const void *Q, const void *K, const void *V,
                          const void *G, const void *dO, void *dQ, void *dK, void *dV, void *ws,
                          size_t ws_bytes, void *stream, StageTimer *tm, float *dG = nullptr)
{
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    if (!general_bwd_supported(pb)) return PSF_ERR_UNSUPPORTED;
    if (!Q || !K || !V || !dO || !dQ || !dK || !dV) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    const bool mfma = bwd_on_mfma(pb);
    const size_t need = mfma ? mfma_bwd_workspace_bytes(pb) : general_bwd_workspace_bytes(pb);
    if (!ws) return PSF_ERR_NULL;
    if (ws_bytes < need) return PSF_ERR_WORKSPACE;
    if (((uintptr_t)ws & 255u) != 0) return PSF_ERR_WORKSPACE;
    if (mfma && !aligned16({Q, K, V, G, dO, dQ, dK, dV})) return PSF_ERR_ALIGNMENT;
    if (dG && !pb.learned) return PSF_ERR_UNSUPPORTED;
    if (mfma) return mfma_attn_bwd(pb, Q, K, V, G, dO, dQ, dK, dV, ws, (hipStream_t)stream, tm, nullptr, nullptr, dG);
    return general_attn_bwd(pb, Q, K, V, G, dO, dQ, dK, dV, ws, (hipStream_t)stream, tm, dG);
}

// ---- scratch of the entry point that allocates nothing ------------------------------------
// One array per GPU the library runs on, held until the process ends.  In host code the
// array's name is only a handle for the symbol, never a device address: the address on the
// current device is asked for once per device and kept; kernels and everything else only
// ever see that pointer.
static __device__ __align__(256) unsigned char scratch[PSF_STATIC_SCRATCH_BYTES];

static const int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void *scratch_ptr[kMaxDevices];            // per device; null until its first call

static psf_status static_scratch(void **out)
{
    int dev = -1;
    PSF_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PSF_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        PSF_HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));   // with `dev` current
        if (!ptr || ((uintptr_t)ptr & 255u) != 0) return PSF_ERR_HIP;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return PSF_OK;
}

}  // namespace psf

using namespace psf;

extern "C" {

psf_status psf_check_desc(const psf_desc *desc)
{
    Problem pb;
    return make_problem(desc, &pb);
}

int psf_kernel_path(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK) return -1;
    return select_path(pb);
}

int psf_fwd_beside_states(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK || select_path(pb) != 1) return 0;
    return mfma_beside_states(pb);
}

size_t psf_g_len(int32_t d, int32_t r, int32_t p)
{
    if (d <= 0 || r <= 0 || p < 4) return 0;
    const size_t half = (size_t)p / 2;
    const size_t n_first = half >= 2 ? half : 0;          // d x r matrices (Theorem 1.1 item 3)
    const size_t n_inner = half >= 4 ? half - 2 : 0;      // r x r matrices
    return n_first * (size_t)d * (size_t)r + n_inner * (size_t)r * (size_t)r;
}

size_t psf_learned_len(int32_t d, int32_t r, int32_t p)
{
    if (d <= 0 || r <= 0 || p < 4) return 0;
    auto net = [&](size_t win) {                          // g1, b1, W1, g2, b2, W2, W3, W4
        const size_t hid = 8 * (size_t)r;
        return 2 * win + win * hid + 2 * hid + hid * r + (size_t)r * hid + hid * r;
    };
    const size_t half = (size_t)p / 2;
    return half * net((size_t)d) + (half >= 4 ? half - 2 : 0) * net((size_t)r);
}

size_t psf_workspace_bytes(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK) return 0;
    return select_path(pb) == 1 ? mfma_workspace_bytes(pb) : general_workspace_bytes(pb);
}

psf_status psf_sketch(const psf_desc *desc, const void *X, const void *G, void *M_out,
                      void *Phi_out, void *hip_stream)
{
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    if (!X) return PSF_ERR_NULL;
    if (!M_out && !Phi_out) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    hipStream_t s = (hipStream_t)hip_stream;
    // This entry point has no workspace, so it always runs the general kernel (fp32
    // arithmetic, any shape); the MFMA sketch lives inside psf_causal_attn_fwd.
    return general_sketch(pb, X, G, M_out, Phi_out, s);
}

psf_status psf_causal_attn_fwd(const psf_desc *desc, const void *Q, const void *K, const void *V,
                               const void *G, void *O, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    return run_attn(desc, Q, K, V, G, O, workspace, workspace_bytes, hip_stream, nullptr);
}

psf_status psf_causal_attn_fwd_static(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                      const void *G, void *O, void *hip_stream)
{
    // sizes first: nothing is touched for a problem that does not fit
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    const size_t need = psf_workspace_bytes(desc);
    if (need > (size_t)PSF_STATIC_SCRATCH_BYTES) return PSF_ERR_WORKSPACE;
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != PSF_OK) return st;
    // every kernel of the forward path writes what it later reads, so the previous call's
    // contents need no clearing
    return run_attn(desc, Q, K, V, G, O, ws, (size_t)PSF_STATIC_SCRATCH_BYTES, hip_stream, nullptr);
}

psf_status psf_causal_attn_fwd_timed(const psf_desc *desc, const void *Q, const void *K,
                                     const void *V, const void *G, void *O, void *workspace,
                                     size_t workspace_bytes, void *hip_stream, float *stage_ms,
                                     int32_t n_stages, int32_t *n_written)
{
    if (!stage_ms || n_stages <= 0) return PSF_ERR_NULL;
    if (n_written) *n_written = 0;
    // validate before creating any event
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    StageTimer tm;
    st = tm.begin((hipStream_t)hip_stream);
    if (st != PSF_OK) return st;
    st = run_attn(desc, Q, K, V, G, O, workspace, workspace_bytes, hip_stream, &tm);
    int w = 0;
    psf_status st2 = tm.finish(stage_ms, n_stages, &w);
    if (n_written) *n_written = w;
    return st != PSF_OK ? st : st2;
}

size_t psf_noncausal_workspace_bytes(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK) return 0;
    return select_path(pb) == 1 ? mfma_noncausal_workspace_bytes(pb) : general_workspace_bytes(pb);
}

psf_status psf_noncausal_attn_fwd(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                  const void *G, void *O, void *workspace, size_t workspace_bytes,
                                  void *hip_stream)
{
    return run_noncausal(desc, Q, K, V, G, O, workspace, workspace_bytes, hip_stream, nullptr);
}

psf_status psf_noncausal_attn_fwd_timed(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                        const void *G, void *O, void *workspace, size_t workspace_bytes,
                                        void *hip_stream, float *stage_ms, int32_t n_stages,
                                        int32_t *n_written)
{
    if (!stage_ms || n_stages <= 0) return PSF_ERR_NULL;
    if (n_written) *n_written = 0;
    Problem pb;
    psf_status st = make_problem(desc, &pb);       // validate before creating any event
    if (st != PSF_OK) return st;
    StageTimer tm;
    st = tm.begin((hipStream_t)hip_stream);
    if (st != PSF_OK) return st;
    st = run_noncausal(desc, Q, K, V, G, O, workspace, workspace_bytes, hip_stream, &tm);
    int w = 0;
    psf_status st2 = tm.finish(stage_ms, n_stages, &w);
    if (n_written) *n_written = w;
    return st != PSF_OK ? st : st2;
}

size_t psf_fwd_save_bytes(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK || !general_bwd_supported(pb) || !bwd_on_mfma(pb)) return 0;
    return mfma_fwd_save_bytes(pb);
}

psf_status psf_causal_attn_fwd_save(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                    const void *G, void *O, void *save, size_t save_bytes, void *hip_stream)
{
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    if (!general_bwd_supported(pb) || !bwd_on_mfma(pb)) return PSF_ERR_UNSUPPORTED;
    if (!Q || !K || !V || !O || !save) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    if (save_bytes < mfma_fwd_save_bytes(pb) || ((uintptr_t)save & 255u) != 0) return PSF_ERR_WORKSPACE;
    if (!aligned16({Q, K, V, G, O})) return PSF_ERR_ALIGNMENT;
    return mfma_attn_fwd_save(pb, Q, K, V, G, O, save, (hipStream_t)hip_stream, nullptr);
}

static psf_status run_bwd_saved(const psf_desc *desc, const void *Q, const void *K, const void *V, const void *G,
                                const void *O, const void *dO, void *dQ, void *dK, void *dV, float *dG, void *save,
                                size_t save_bytes, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Problem pb;
    psf_status st = make_problem(desc, &pb);
    if (st != PSF_OK) return st;
    if (!general_bwd_supported(pb) || !bwd_on_mfma(pb)) return PSF_ERR_UNSUPPORTED;
    if (dG && !pb.learned) return PSF_ERR_UNSUPPORTED;
    if (!Q || !K || !V || !O || !dO || !dQ || !dK || !dV || !save || !workspace) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    if (save_bytes < mfma_fwd_save_bytes(pb) || ((uintptr_t)save & 255u) != 0) return PSF_ERR_WORKSPACE;
    if (workspace_bytes < mfma_bwd_workspace_bytes(pb) || ((uintptr_t)workspace & 255u) != 0) return PSF_ERR_WORKSPACE;
    if (!aligned16({Q, K, V, G, O, dO, dQ, dK, dV})) return PSF_ERR_ALIGNMENT;
    return mfma_attn_bwd(pb, Q, K, V, G, dO, dQ, dK, dV, workspace, (hipStream_t)hip_stream, nullptr, save, O, dG);
}

psf_status psf_causal_attn_bwd_saved(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                     const void *G, const void *O, const void *dO, void *dQ, void *dK,
                                     void *dV, void *save, size_t save_bytes, void *workspace,
                                     size_t workspace_bytes, void *hip_stream)
{
    return run_bwd_saved(desc, Q, K, V, G, O, dO, dQ, dK, dV, nullptr, save, save_bytes, workspace, workspace_bytes,
                         hip_stream);
}

psf_status psf_causal_attn_bwd_saved_learned(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                             const void *G, const void *O, const void *dO, void *dQ, void *dK,
                                             void *dV, float *dG, void *save, size_t save_bytes, void *workspace,
                                             size_t workspace_bytes, void *hip_stream)
{
    if (!dG) return PSF_ERR_NULL;
    return run_bwd_saved(desc, Q, K, V, G, O, dO, dQ, dK, dV, dG, save, save_bytes, workspace, workspace_bytes,
                         hip_stream);
}

int psf_bwd_kernel_path(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK || !general_bwd_supported(pb)) return -1;
    return bwd_on_mfma(pb) ? 3 : 2;
}

size_t psf_bwd_workspace_bytes(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK || !general_bwd_supported(pb)) return 0;
    return bwd_on_mfma(pb) ? mfma_bwd_workspace_bytes(pb) : general_bwd_workspace_bytes(pb);
}

psf_status psf_causal_attn_bwd(const psf_desc *desc, const void *Q, const void *K, const void *V,
                               const void *G, const void *dO, void *dQ, void *dK, void *dV,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return run_bwd(desc, Q, K, V, G, dO, dQ, dK, dV, workspace, workspace_bytes, hip_stream, nullptr);
}

psf_status psf_causal_attn_bwd_learned(const psf_desc *desc, const void *Q, const void *K, const void *V,
                                       const void *G, const void *dO, void *dQ, void *dK, void *dV,
                                       float *dG, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!dG) return PSF_ERR_NULL;
    return run_bwd(desc, Q, K, V, G, dO, dQ, dK, dV, workspace, workspace_bytes, hip_stream, nullptr, dG);
}

psf_status psf_causal_attn_bwd_timed(const psf_desc *desc, const void *Q, const void *K,
                                     const void *V, const void *G, const void *dO, void *dQ,
                                     void *dK, void *dV, void *workspace, size_t workspace_bytes,
                                     void *hip_stream, float *stage_ms, int32_t n_stages,
                                     int32_t *n_written)
{
    if (!stage_ms || n_stages <= 0) return PSF_ERR_NULL;
    if (n_written) *n_written = 0;
    Problem pb;
    psf_status st = make_problem(desc, &pb);       // validate before creating any event
    if (st != PSF_OK) return st;
    if (!general_bwd_supported(pb)) return PSF_ERR_UNSUPPORTED;
    StageTimer tm;
    st = tm.begin((hipStream_t)hip_stream);
    if (st != PSF_OK) return st;
    st = run_bwd(desc, Q, K, V, G, dO, dQ, dK, dV, workspace, workspace_bytes, hip_stream, &tm);
    int w = 0;
    psf_status st2 = tm.finish(stage_ms, n_stages, &w);
    if (n_written) *n_written = w;
    return st != PSF_OK ? st : st2;
}

size_t psf_decode_state_bytes(const psf_desc *desc)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK || !decode_supported(pb)) return 0;
    return decode_state_bytes(pb);
}

static psf_status decode_check(const psf_desc *desc, Problem *pb, const void *state, size_t state_bytes)
{
    psf_status st = make_problem(desc, pb);
    if (st != PSF_OK) return st;
    if (!decode_supported(*pb)) return PSF_ERR_UNSUPPORTED;
    if (!state) return PSF_ERR_NULL;
    if (state_bytes < decode_state_bytes(*pb) || ((uintptr_t)state & 255u) != 0) return PSF_ERR_WORKSPACE;
    return PSF_OK;
}

psf_status psf_decode_reset(const psf_desc *desc, void *state, size_t state_bytes, void *hip_stream)
{
    Problem pb;
    psf_status st = decode_check(desc, &pb, state, state_bytes);
    if (st != PSF_OK) return st;
    return decode_reset(pb, state, (hipStream_t)hip_stream);
}

psf_status psf_decode_step(const psf_desc *desc, const void *q, const void *k, const void *v,
                           const void *G, int32_t pos, void *state, size_t state_bytes, void *o,
                           void *hip_stream)
{
    Problem pb;
    psf_status st = decode_check(desc, &pb, state, state_bytes);
    if (st != PSF_OK) return st;
    if (!q || !k || !v || !o) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    if (pos < 0 || pos >= pb.n) return PSF_ERR_SHAPE;
    return decode_step(pb, q, k, v, G, pos, state, o, (hipStream_t)hip_stream);
}

size_t psf_decode_prefill_workspace_bytes(const psf_desc *desc, int32_t n_prompt)
{
    Problem pb;
    if (make_problem(desc, &pb) != PSF_OK || !decode_supported(pb) || n_prompt < 0 || n_prompt > pb.n) return 0;
    return decode_prefill_workspace_bytes(pb, n_prompt);
}

psf_status psf_decode_prefill(const psf_desc *desc, const void *K, const void *V, const void *G,
                              int32_t n_prompt, void *state, size_t state_bytes, void *workspace,
                              size_t workspace_bytes, void *hip_stream)
{
    Problem pb;
    psf_status st = decode_check(desc, &pb, state, state_bytes);
    if (st != PSF_OK) return st;
    if (n_prompt < 0 || n_prompt > pb.n) return PSF_ERR_SHAPE;
    if (n_prompt > 0 && (!K || !V)) return PSF_ERR_NULL;
    if (pb.g_len > 0 && !G) return PSF_ERR_NULL;
    const size_t need = decode_prefill_workspace_bytes(pb, n_prompt);
    if (need > 0 && !workspace) return PSF_ERR_NULL;
    if (workspace_bytes < need || (need > 0 && ((uintptr_t)workspace & 255u) != 0)) return PSF_ERR_WORKSPACE;
    // (the hand-over has its own rule for when the forward pass's MFMA kernels take the complete
    // blocks of the prompt: it does not depend on b % 256 or on the in-block rule)
    if (decode_prefill_uses_mfma(pb, n_prompt) && !aligned16({K, V, G})) return PSF_ERR_ALIGNMENT;
    return decode_prefill(pb, K, V, G, n_prompt, state, workspace, (hipStream_t)hip_stream);
}

const char *psf_stage_name(int path, int32_t stage)
{
    static const char *bwd[] = {"sketches", "forward_rows", "reverse_states", "query_side",
                                "key_side", "sketch_gradient"};
    if (path == 2 && stage >= 0 && stage < 6) return bwd[stage];
    // (learned sketches: the last stage also holds the networks' reverse pass and the parameter sums)
    static const char *bwd_mfma[] = {"forward_again", "g_c_and_layouts", "mirror_states", "in_block_and_dv",
                                     "cross_block_and_sketch_gradient"};
    if (path == 3 && stage >= 0 && stage < 5) return bwd_mfma[stage];
    static const char *general[] = {"sketch_q", "sketch_k", "block_states", "exclusive_scan",
                                    "output"};
    static const char *mfma[] = {"sketch_and_layouts", "denominator_scan", "block_states_scan",
                                 "output"};
    if (path == 0 && stage >= 0 && stage < 5) return general[stage];
    if (path == 1 && stage >= 0 && stage < 4) return mfma[stage];
    return "";
}

const char *psf_status_string(psf_status status)
{
    switch (status) {
    case PSF_OK: return "ok";
    case PSF_ERR_NULL: return "required pointer is NULL";
    case PSF_ERR_SHAPE: return "invalid shape (non-positive size or n not a multiple of b)";
    case PSF_ERR_UNSUPPORTED: return "unsupported parameter";
    case PSF_ERR_WORKSPACE: return "workspace too small or misaligned";
    case PSF_ERR_ALIGNMENT: return "tensor not 16-byte aligned for the bf16 MFMA kernels";
    case PSF_ERR_HIP: return "HIP call or kernel launch failed";
    }
    return "unknown status";
}

}  // extern "C"
