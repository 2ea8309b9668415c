// Internal declarations shared by the translation units of libpsf (not part of the ABI).
#ifndef PSF_INTERNAL_H
#define PSF_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "psf.h"

namespace psf {

// Host-side view of a validated descriptor.
struct Problem {
    int batch, heads, units;
    int n, d, dv, p, r, b, t;
    int mcols;        // columns of m(x): r, or d when p == 2 (Algorithm 1 base case)
    long long F;      // explicit feature count: mcols^2, or d^p with exact features
    bool bf16, exact_feat, local_exact, per_head, learned;
    size_t g_len;     // entries of one set of sketch matrices
};

psf_status make_problem(const psf_desc *desc, Problem *out);
int select_path(const Problem &pb);

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Event recorder used by the timed entry point; inert when `on` is false.
struct StageTimer {
    bool on = false;
    hipStream_t stream = nullptr;
    static const int kMax = 12;
    hipEvent_t ev[kMax + 1];
    int count = 0;
    psf_status begin(hipStream_t s);
    void mark();                       // closes the current stage
    psf_status finish(float *ms, int cap, int *written);
};

// General fp32 path (any descriptor the check admits).
size_t general_workspace_bytes(const Problem &pb);
psf_status general_sketch(const Problem &pb, const void *X, const void *G, void *M_out,
                          void *Phi_out, hipStream_t s);
// noncausal: Section 2.2 (every query sees every key; b only partitions the work).
psf_status general_attn(const Problem &pb, const void *Q, const void *K, const void *V,
                        const void *G, void *O, void *ws, hipStream_t s, StageTimer *tm,
                        bool noncausal = false);

// m(x) of every row as fp32 [rows][mcols] (general sketch kernel).
psf_status general_sketch_f32(const Problem &pb, const void *X, const void *G, float *M_f32,
                              hipStream_t s);
// The same for two sets of rows (X -> M_f32, X2 -> M2_f32) in one launch.
psf_status general_sketch_pair_f32(const Problem &pb, const void *X, const void *X2, const void *G,
                                   float *M_f32, float *M2_f32, hipStream_t s);

// Backward pass (general fp32 kernels; sketch features only).  dG: with learned sketches,
// the gradient with respect to the networks' parameters (fp32 [sets][g_len], overwritten), or null.
bool general_bwd_supported(const Problem &pb);
size_t general_bwd_workspace_bytes(const Problem &pb);
psf_status general_attn_bwd(const Problem &pb, const void *Q, const void *K, const void *V,
                            const void *G, const void *dO, void *dQ, void *dK, void *dV, void *ws,
                            hipStream_t s, StageTimer *tm, float *dG = nullptr);

psf_status general_sketch_bwd(const Problem &pb, const void *X, const void *G, const float *dM,
                              const float *direct, void *dX, hipStream_t s);

// Backward pass on MFMA (bf16, d = dv in {64, 128}, p in {4, 8}, r in {32, 64}, b % 256 == 0, exact
// in-block weights; for d = 64 and p = 4 also Section 3.1's in-block rule (r = 64) and learned sketches).
bool mfma_bwd_supported(const Problem &pb);
size_t mfma_bwd_workspace_bytes(const Problem &pb);
// saved / O_saved: what mfma_attn_fwd_save left and the output it wrote (skips the forward pass
// inside; random sketches only), or null.  dG (learned sketches only): fp32 [sets][g_len], the
// gradient of the network parameters, or null to treat them as constants.
psf_status mfma_attn_bwd(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                         const void *dO, void *dQ, void *dK, void *dV, void *ws, hipStream_t s,
                         StageTimer *tm, void *saved = nullptr, const void *O_saved = nullptr,
                         float *dG = nullptr);
size_t mfma_fwd_save_bytes(const Problem &pb);
psf_status mfma_attn_fwd_save(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                              void *O, void *saved, hipStream_t s, StageTimer *tm);

// Token-by-token evaluation (fp32 kernels; sketch features only).
bool decode_supported(const Problem &pb);
size_t decode_state_bytes(const Problem &pb);
psf_status decode_reset(const Problem &pb, void *state, hipStream_t s);
psf_status decode_step(const Problem &pb, const void *q, const void *k, const void *v, const void *G,
                       int pos, void *state, void *o, hipStream_t s);
// State after the first n_prompt tokens (K, V: [units][n_prompt][d | dv]), as if they had been fed
// one by one; ws: decode_prefill_workspace_bytes.
size_t decode_prefill_workspace_bytes(const Problem &pb, int n_prompt);
// true when the complete blocks of the prompt go through the forward path's bf16 MFMA kernels
// (which move the caller's K, V, G in 16-byte pieces)
bool decode_prefill_uses_mfma(const Problem &pb, int n_prompt);
psf_status decode_prefill(const Problem &pb, const void *K, const void *V, const void *G, int n_prompt,
                          void *state, void *ws, hipStream_t s);

// bf16 MFMA path.
size_t mfma_workspace_bytes(const Problem &pb);
int mfma_beside_states(const Problem &pb);
psf_status mfma_attn(const Problem &pb, const void *Q, const void *K, const void *V,
                     const void *G, void *O, void *ws, hipStream_t s, StageTimer *tm);
// Sum over n_tok tokens per unit (K, V contiguous [units][n_tok][d]) of phi'(k) v^T, in the output
// kernel's state layout ([a][b'/8][c][8] bf16; b' > a doubled, b' < a zero), and the fp32
// partial sums of m(k)^T m(k) ([units][parts][r][r]); for the decode hand-over.
bool mfma_total_state_supported(const Problem &pb, int n_tok);
size_t mfma_total_state_workspace_bytes(const Problem &pb, int n_tok);
psf_status mfma_total_state(const Problem &pb, int n_tok, const void *K, const void *V, const void *G, void *ws,
                            hipStream_t s, const void **Zg, const float **Spart, int *parts_per_unit);
size_t mfma_noncausal_workspace_bytes(const Problem &pb);
psf_status mfma_attn_noncausal(const Problem &pb, const void *Q, const void *K, const void *V,
                               const void *G, void *O, void *ws, hipStream_t s, StageTimer *tm);

#define PSF_HIP_TRY(expr)                                   \
    do {                                                    \
        hipError_t e__ = (expr);                            \
        if (e__ != hipSuccess) return PSF_ERR_HIP;          \
    } while (0)

#define PSF_LAUNCH_CHECK()                                  \
    do {                                                    \
        if (hipGetLastError() != hipSuccess) return PSF_ERR_HIP; \
    } while (0)

// ---- storage helpers (device) ------------------------------------------------------
typedef uint16_t bf16_t;   // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float load_f(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_f(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void store_f(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_f(bf16_t *p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// ---- Algorithm 1 for a few rows (device) ----------------------------------------------
// m(x) = PolySketchWithNegativity(x, r, p / 2) of NR rows xs[i][0 .. d) held in LDS, computed by
// a workgroup of kSketchThreads threads that all call this (it contains barriers); the rows
// share g_set, the set of sketch matrices of their head (p / 2 of d x r, then the r x r ones
// level by level), so every matrix entry is loaded once for all of them.  fin[i] receives the
// LDS address of the r results of row i (inside the scratch; xs[i] itself for p == 2), valid
// after the barrier this function ends with.  Thread (col, part) sums the input rows
// e = part, part + nparts, ... of both projections of a node; the partial sums are then added
// in a fixed order.
constexpr int kSketchThreads = 256;
template <int NR>
struct SketchScratchN {
    float lev[NR][2][4][PSF_MAX_DIM];
    float pu[NR][kSketchThreads], pv[NR][kSketchThreads];
};
typedef SketchScratchN<1> SketchScratch;

template <typename T, int NR>
__device__ __forceinline__ void sketch_rows_lds(const float *const (&xs)[NR], const T *g_set, int d, int r, int p,
                                                SketchScratchN<NR> &sc_lds, const float *(&fin)[NR])
{
    if (p <= 2) {
#pragma unroll
        for (int i = 0; i < NR; ++i) fin[i] = xs[i];
        return;
    }
    const int tid = threadIdx.x;
    const T *g_inner = g_set + (size_t)(p / 2) * d * r;
    const float sc = sqrtf(1.0f / (float)r);
    int cur = 0, count = p / 4;                       // degree-2 sketches of x
    const int nparts = kSketchThreads / r > 0 ? kSketchThreads / r : 1, part = tid / r, col = tid % r;
    for (int j = 0; j < count; ++j) {
        const T *ga = g_set + (size_t)(2 * j) * d * r;
        const T *gb = ga + (size_t)d * r;
        float u[NR], v[NR];
#pragma unroll
        for (int i = 0; i < NR; ++i) u[i] = v[i] = 0.f;
        if (part < nparts && col < r) {
            for (int e = part; e < d; e += nparts) {
                const float a = load_f(ga, (size_t)e * r + col), b = load_f(gb, (size_t)e * r + col);
#pragma unroll
                for (int i = 0; i < NR; ++i) {
                    u[i] += xs[i][e] * a;
                    v[i] += xs[i][e] * b;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            sc_lds.pu[i][tid] = u[i];
            sc_lds.pv[i][tid] = v[i];
        }
        __syncthreads();
        if (tid < r) {
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                float us = 0.f, vs = 0.f;
                for (int q2 = 0; q2 < nparts; ++q2) { us += sc_lds.pu[i][q2 * r + tid]; vs += sc_lds.pv[i][q2 * r + tid]; }
                sc_lds.lev[i][cur][j][tid] = sc * (us * vs);
            }
        }
    }
    __syncthreads();
    size_t inner_at = 0;                              // r x r matrices, level by level
    while (count > 1) {
        const int next = count / 2;
        if (tid < r) {
            for (int j = 0; j < next; ++j) {
                const T *ga = g_inner + (inner_at + 2 * j) * (size_t)r * r;
                const T *gb = ga + (size_t)r * r;
                float u[NR], v[NR];
#pragma unroll
                for (int i = 0; i < NR; ++i) u[i] = v[i] = 0.f;
                for (int e = 0; e < r; ++e) {
                    const float a = load_f(ga, (size_t)e * r + tid), b = load_f(gb, (size_t)e * r + tid);
#pragma unroll
                    for (int i = 0; i < NR; ++i) {
                        u[i] += sc_lds.lev[i][cur][2 * j][e] * a;
                        v[i] += sc_lds.lev[i][cur][2 * j + 1][e] * b;
                    }
                }
#pragma unroll
                for (int i = 0; i < NR; ++i) sc_lds.lev[i][cur ^ 1][j][tid] = sc * (u[i] * v[i]);
            }
        }
        __syncthreads();
        inner_at += 2 * (size_t)next;
        count = next;
        cur ^= 1;
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) fin[i] = sc_lds.lev[i][cur][0];
}

template <typename T>
__device__ __forceinline__ const float *sketch_row_lds(const float *xs, const T *g_set, int d, int r, int p,
                                                       SketchScratch &sc_lds)
{
    const float *const rows[1] = {xs};
    const float *fin[1];
    sketch_rows_lds<T, 1>(rows, g_set, d, r, p, sc_lds, fin);
    return fin[0];
}

}  // namespace psf
#endif
