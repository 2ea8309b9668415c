// General fp32 path of libpsf: every descriptor the check admits (any d, dv, r <= 256,
// p in {2,4,8,16}, exact features x^{(x)p}, either in-block rule, fp32 or bf16 storage).
// Plain LDS-staged VALU kernels that follow the block algorithm of PolySketchFormer
// (arXiv 2310.01655, Sections 3.1 and 3.2) step by step; the tuned bf16 MFMA kernels for
// the large shapes live in psf_mfma.hip.
#include "psf_internal.h"

namespace psf {
namespace {

constexpr int kThreads = 256;
constexpr int kStateFeat = 8;     // features per workgroup in the block-state kernel
constexpr int kStateChunk = 64;   // tokens staged per step in the block-state kernel
constexpr int kOutRows = 8;       // rows per workgroup in the output kernel (at most)
constexpr int kOutChunk = 512;    // features / keys staged per step in the output kernel

__device__ __forceinline__ float pow_pow2(float x, int p)
{
    for (int e = 1; e < p; e <<= 1) x *= x;      // p is a power of two: repeated squaring
    return x;
}

// phi(x)[f] for exact features: f = (a_1 ... a_p) in base d, most significant first
// (x^{(x)p} = x (x) x^{(x)(p-1)}, Section 1.2), value prod_e x[a_e].
template <typename T>
__device__ __forceinline__ float exact_feature(const T *x, long long f, int d, int p)
{
    float v = 1.f;
    for (int e = 0; e < p; ++e) {
        v *= load_f(x, (size_t)(f % d));
        f /= d;
    }
    return v;
}

// ---- Algorithm 1 for one row per loop iteration; intermediates live in LDS ----------
template <typename T>
__global__ __launch_bounds__(kThreads) void gen_sketch_kernel(
    const T *__restrict__ X, const T *__restrict__ G, long long rows, int n, int heads,
    int per_head, int d, int r, int p, int exact, long long F, size_t g_len,
    float *__restrict__ M_f32, T *__restrict__ M_st, T *__restrict__ Phi,
    const T *__restrict__ X2, float *__restrict__ M2_f32)
{
    // X2 / M2_f32 (optional): a second set of `rows` rows sketched by the same launch (fp32 out only)
    static_assert(kThreads == kSketchThreads, "sketch_row_lds assumes this workgroup size");
    __shared__ float xs[PSF_MAX_DIM];
    __shared__ SketchScratch scratch;
    const int tid = threadIdx.x;
    const int mcols = (p == 2) ? d : r;
    const long long total = X2 ? 2 * rows : rows;
    for (long long row_all = blockIdx.x; row_all < total; row_all += gridDim.x) {
        const bool second = row_all >= rows;
        const long long row = second ? row_all - rows : row_all;
        const T *x = (second ? X2 : X) + (size_t)row * d;
        __syncthreads();
        if (tid < d) xs[tid] = load_f(x, tid);
        __syncthreads();
        const float *fin = xs;
        if (!exact && p > 2) {
            const int head = (int)((row / n) % heads);
            fin = sketch_row_lds(xs, G + (per_head ? (size_t)head * g_len : 0), d, r, p, scratch);
        }
        if (!exact) {
            if (second) {
                if (tid < mcols) M2_f32[(size_t)row * mcols + tid] = fin[tid];
                continue;
            }
            if (tid < mcols) {
                if (M_f32) M_f32[(size_t)row * mcols + tid] = fin[tid];
                if (M_st) store_f(M_st, (size_t)row * mcols + tid, fin[tid]);
            }
            if (Phi)
                for (int idx = tid; idx < mcols * mcols; idx += kThreads)
                    store_f(Phi, (size_t)row * F + idx, fin[idx / mcols] * fin[idx % mcols]);
        } else if (Phi) {
            for (long long f = tid; f < F; f += kThreads) {
                long long g = f;                 // the product does not depend on digit order
                float v = 1.f;
                for (int e = 0; e < p; ++e) { v *= xs[g % d]; g /= d; }
                store_f(Phi, (size_t)row * F + f, v);
            }
        }
    }
}

// ---- Algorithm 2 (learnable sketches, Appendix D), one row per loop iteration -------------
// Every projection M G of Algorithm 1 becomes a dense network f(M); the node returns
// sqrt(r) tanh(sqrt(1/r) f1(M1) * f2(M2)).  The reading of the appendix (layer order, no dense
// biases, layer-norm eps, tanh form of gelu, parameter order) is stated in include/psf.h.
constexpr int kMaxHidden = 8 * PSF_MAX_DIM;

__device__ __forceinline__ float gelu_tanh(float x)
{
    return 0.5f * x * (1.0f + tanhf(0.7978845608028654f * (x + 0.044715f * x * x * x)));
}

// out[e] = (x[e] - mean) / sqrt(var + eps) * g[e] + b[e], e < m; x, out in LDS (may alias);
// red is kThreads + 2 floats of LDS.
template <typename T>
__device__ void wg_layer_norm(const float *x, int m, const T *g, const T *b, float *out, float *red)
{
    const int tid = threadIdx.x;
    float s = 0.f;
    for (int e = tid; e < m; e += kThreads) s += x[e];
    red[tid] = s;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int q = 0; q < kThreads; ++q) t += red[q];
        red[kThreads] = t / (float)m;
    }
    __syncthreads();
    const float mean = red[kThreads];
    s = 0.f;
    for (int e = tid; e < m; e += kThreads) s += (x[e] - mean) * (x[e] - mean);
    __syncthreads();
    red[tid] = s;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int q = 0; q < kThreads; ++q) t += red[q];
        red[kThreads + 1] = rsqrtf(t / (float)m + 1e-6f);
    }
    __syncthreads();
    const float inv = red[kThreads + 1];
    for (int e = tid; e < m; e += kThreads) out[e] = (x[e] - mean) * inv * load_f(g, e) + load_f(b, e);
    __syncthreads();
}

// out[c] = act(sum_e x[e] W[e * cols + c]) for c < cols; x, out in LDS (must not alias)
template <typename T, bool GELU>
__device__ void wg_dense(const float *x, int rows, const T *W, int cols, float *out)
{
    for (int c = threadIdx.x; c < cols; c += kThreads) {
        float s = 0.f;
        for (int e = 0; e < rows; ++e) s += x[e] * load_f(W, (size_t)e * cols + c);
        out[c] = GELU ? gelu_tanh(s) : s;
    }
    __syncthreads();
}

// one network: inp (LDS, win) -> out (LDS, r); P points at its parameters
template <typename T>
__device__ void wg_learned_net(const float *inp, int win, int r, const T *P, float *out, float *u,
                               float *h, float *red)
{
    const int hid = 8 * r;
    const T *g1 = P, *b1 = g1 + win, *W1 = b1 + win;
    const T *g2 = W1 + (size_t)win * hid, *b2 = g2 + hid, *W2 = b2 + hid;
    const T *W3 = W2 + (size_t)hid * r, *W4 = W3 + (size_t)r * hid;
    wg_layer_norm(inp, win, g1, b1, u, red);
    wg_dense<T, true>(u, win, W1, hid, h);
    wg_layer_norm(h, hid, g2, b2, h, red);
    wg_dense<T, false>(h, hid, W2, r, u);
    wg_dense<T, true>(u, r, W3, hid, h);
    wg_dense<T, false>(h, hid, W4, r, out);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void gen_sketch_learned_kernel(
    const T *__restrict__ X, const T *__restrict__ P, long long rows, int n, int heads, int per_head,
    int d, int r, int p, size_t p_len, float *__restrict__ M_f32, T *__restrict__ M_st,
    T *__restrict__ Phi, const T *__restrict__ X2, float *__restrict__ M2_f32)
{
    // X2 / M2_f32 (optional): a second set of `rows` rows sketched by the same launch (fp32 out only)
    __shared__ float xs[PSF_MAX_DIM], u[kMaxHidden], h[kMaxHidden], red[kThreads + 2];
    __shared__ float f1[PSF_MAX_DIM], f2[PSF_MAX_DIM], m1[PSF_MAX_DIM], m2[PSF_MAX_DIM];
    const int tid = threadIdx.x;
    const size_t len_d = 2 * (size_t)d + (size_t)d * 8 * r + 16 * (size_t)r + 24 * (size_t)r * r;
    const float sr = sqrtf((float)r);
    const long long total = X2 ? 2 * rows : rows;
    for (long long row_all = blockIdx.x; row_all < total; row_all += gridDim.x) {
        const bool second = row_all >= rows;
        const long long row = second ? row_all - rows : row_all;
        __syncthreads();
        if (tid < d) xs[tid] = load_f(second ? X2 : X, (size_t)row * d + tid);
        __syncthreads();
        const int head = (int)((row / n) % heads);
        const T *P0 = P + (per_head ? (size_t)head * p_len : 0);
        // first-level node 0: networks 0 and 1 on x
        wg_learned_net(xs, d, r, P0, f1, u, h, red);
        wg_learned_net(xs, d, r, P0 + len_d, f2, u, h, red);
        if (tid < r) m1[tid] = sr * tanhf(f1[tid] * f2[tid] / sr);
        __syncthreads();
        if (p == 8) {                                     // second first-level node, then the root
            wg_learned_net(xs, d, r, P0 + 2 * len_d, f1, u, h, red);
            wg_learned_net(xs, d, r, P0 + 3 * len_d, f2, u, h, red);
            if (tid < r) m2[tid] = sr * tanhf(f1[tid] * f2[tid] / sr);
            __syncthreads();
            const size_t len_r = 2 * (size_t)r + (size_t)r * 8 * r + 16 * (size_t)r + 24 * (size_t)r * r;
            wg_learned_net(m1, r, r, P0 + 4 * len_d, f1, u, h, red);
            wg_learned_net(m2, r, r, P0 + 4 * len_d + len_r, f2, u, h, red);
            if (tid < r) m1[tid] = sr * tanhf(f1[tid] * f2[tid] / sr);
            __syncthreads();
        }
        if (second) {
            if (tid < r) M2_f32[(size_t)row * r + tid] = m1[tid];
            continue;
        }
        if (tid < r) {
            if (M_f32) M_f32[(size_t)row * r + tid] = m1[tid];
            if (M_st) store_f(M_st, (size_t)row * r + tid, m1[tid]);
        }
        if (Phi)
            for (int idx = tid; idx < r * r; idx += kThreads)
                store_f(Phi, (size_t)row * r * r + idx, m1[idx / r] * m1[idx % r]);
    }
}

// ---- H_l = phi(K_l)^T [V_l | 1]  (Section 3.1), one block l per blockIdx.y ----------
template <typename T>
__global__ __launch_bounds__(kThreads) void gen_state_kernel(
    const float *__restrict__ MK, const T *__restrict__ K, const T *__restrict__ V,
    float *__restrict__ Z, int n, int d, int dv, int p, int b, int t, int mcols, long long F,
    int exact)
{
    __shared__ float phi[kStateChunk][kStateFeat];
    const int tid = threadIdx.x, l = blockIdx.y, u = blockIdx.z;
    const long long f0 = (long long)blockIdx.x * kStateFeat;
    const int kc = dv + 1;
    float acc[kStateFeat][2];
    for (int ff = 0; ff < kStateFeat; ++ff) acc[ff][0] = acc[ff][1] = 0.f;
    const size_t row0 = (size_t)u * n + (size_t)l * b;
    for (int j0 = 0; j0 < b; j0 += kStateChunk) {
        __syncthreads();
        for (int idx = tid; idx < kStateChunk * kStateFeat; idx += kThreads) {
            const int jj = idx / kStateFeat, ff = idx % kStateFeat;
            float v = 0.f;
            if (j0 + jj < b && f0 + ff < F) {
                const size_t row = row0 + j0 + jj;
                const long long f = f0 + ff;
                v = exact ? exact_feature(K + row * d, f, d, p)
                          : MK[row * mcols + f / mcols] * MK[row * mcols + f % mcols];
            }
            phi[jj][ff] = v;
        }
        __syncthreads();
        const int lim = min(kStateChunk, b - j0);
        for (int ci = 0; ci < 2; ++ci) {
            const int c = tid + ci * kThreads;
            if (c >= kc) break;
            for (int jj = 0; jj < lim; ++jj) {
                const float v = (c < dv) ? load_f(V, (row0 + j0 + jj) * dv + c) : 1.f;
                for (int ff = 0; ff < kStateFeat; ++ff) acc[ff][ci] += phi[jj][ff] * v;
            }
        }
    }
    float *z = Z + (((size_t)u * t + l) * (size_t)F) * kc;
    for (int ci = 0; ci < 2; ++ci) {
        const int c = tid + ci * kThreads;
        if (c >= kc) break;
        for (int ff = 0; ff < kStateFeat; ++ff)
            if (f0 + ff < F) z[(size_t)(f0 + ff) * kc + c] = acc[ff][ci];
    }
}

// ---- Z_l = sum_{j<l} H_j, sequential over blocks as in the paper; in place --------------
__global__ __launch_bounds__(kThreads) void gen_scan_kernel(float *__restrict__ Z, int units, int t,
                                                            size_t per_block)
{
    const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= (size_t)units * per_block) return;
    const size_t u = idx / per_block, e = idx % per_block;
    float *z = Z + u * (size_t)t * per_block + e;
    float run = 0.f;
    for (int l = 0; l < t; ++l) {
        const float h = (l < t - 1) ? z[(size_t)l * per_block] : 0.f;   // H_t is never needed
        z[(size_t)l * per_block] = run;
        run += h;
    }
}

// ---- non-causal attention (Section 2.2): one state for all keys, sum of every H_l, in slot 0 ----
__global__ __launch_bounds__(kThreads) void gen_total_kernel(float *__restrict__ Z, int units, int t,
                                                             size_t per_block)
{
    const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= (size_t)units * per_block) return;
    const size_t u = idx / per_block, e = idx % per_block;
    float *z = Z + u * (size_t)t * per_block + e;
    float run = 0.f;
    for (int l = 0; l < t; ++l) run += z[(size_t)l * per_block];
    z[0] = run;
}

// ---- rows of the output: P_l row + phi(q_i)^T Z_l, then divide by 1 + last column ---------
// noncausal: every row takes phi(q_i)^T Z with the one state in slot 0 and has no in-block part
template <typename T>
__global__ __launch_bounds__(kThreads) void gen_out_kernel(
    const float *__restrict__ MQ, const float *__restrict__ MK, const T *__restrict__ Q,
    const T *__restrict__ K, const T *__restrict__ V, const float *__restrict__ Z,
    T *__restrict__ O, int n, int d, int dv, int p, int b, int t, int mcols, long long F,
    int exact_feat, int local_exact, int rows_per_wg, int noncausal)
{
    __shared__ float stage[kOutRows][kOutChunk];
    __shared__ float den_s[kOutRows];
    const int tid = threadIdx.x, u = blockIdx.y;
    const int i0 = blockIdx.x * rows_per_wg;            // first row of this workgroup
    const int l = i0 / b;                               // all its rows lie in block l
    const int kc = dv + 1, RT = rows_per_wg;
    float acc[kOutRows][2];
    for (int rt = 0; rt < kOutRows; ++rt) acc[rt][0] = acc[rt][1] = 0.f;
    const size_t urow = (size_t)u * n;

    if (l > 0 || noncausal) {                           // a_i^T Z_l
        const float *z = Z + (((size_t)u * t + (noncausal ? 0 : l)) * (size_t)F) * kc;
        for (long long f0 = 0; f0 < F; f0 += kOutChunk) {
            __syncthreads();
            for (int idx = tid; idx < RT * kOutChunk; idx += kThreads) {
                const int rt = idx / kOutChunk, ff = idx % kOutChunk;
                const long long f = f0 + ff;
                float v = 0.f;
                if (f < F) {
                    const size_t row = urow + i0 + rt;
                    v = exact_feat ? exact_feature(Q + row * d, f, d, p)
                                   : MQ[row * mcols + f / mcols] * MQ[row * mcols + f % mcols];
                }
                stage[rt][ff] = v;
            }
            __syncthreads();
            const int lim = (int)min((long long)kOutChunk, F - f0);
            for (int ci = 0; ci < 2; ++ci) {
                const int c = tid + ci * kThreads;
                if (c >= kc) break;
                for (int ff = 0; ff < lim; ++ff) {
                    const float zv = z[(size_t)(f0 + ff) * kc + c];
                    for (int rt = 0; rt < kOutRows; ++rt)
                        if (rt < RT) acc[rt][ci] += stage[rt][ff] * zv;
                }
            }
        }
    }

    const int jbeg = l * b, jend = noncausal ? jbeg : i0 + RT;   // keys jbeg .. i0+RT-1 (row rt keeps j <= i0+rt)
    for (int j0 = jbeg; j0 < jend; j0 += kOutChunk) {   // row of P_l = lt(.) [V_l | 1]
        __syncthreads();
        for (int idx = tid; idx < RT * kOutChunk; idx += kThreads) {
            const int rt = idx / kOutChunk, jj = idx % kOutChunk;
            const int j = j0 + jj, i = i0 + rt;
            float w = 0.f;
            if (j <= i) {
                if (local_exact) {
                    const T *q = Q + (urow + i) * d, *k = K + (urow + j) * d;
                    float s = 0.f;
                    for (int e = 0; e < d; ++e) s += load_f(q, e) * load_f(k, e);
                    w = pow_pow2(s, p);
                } else {
                    const float *q = MQ + (urow + i) * mcols, *k = MK + (urow + j) * mcols;
                    float s = 0.f;
                    for (int e = 0; e < mcols; ++e) s += q[e] * k[e];
                    w = s * s;
                }
            }
            stage[rt][jj] = w;
        }
        __syncthreads();
        const int lim = min(kOutChunk, jend - j0);
        for (int ci = 0; ci < 2; ++ci) {
            const int c = tid + ci * kThreads;
            if (c >= kc) break;
            for (int jj = 0; jj < lim; ++jj) {
                const float v = (c < dv) ? load_f(V, (urow + j0 + jj) * dv + c) : 1.f;
                for (int rt = 0; rt < kOutRows; ++rt)
                    if (rt < RT) acc[rt][ci] += stage[rt][jj] * v;
            }
        }
    }

    __syncthreads();
    if (tid == dv % kThreads)
        for (int rt = 0; rt < kOutRows; ++rt)
            if (rt < RT) den_s[rt] = 1.f + acc[rt][dv / kThreads];
    __syncthreads();
    for (int ci = 0; ci < 2; ++ci) {
        const int c = tid + ci * kThreads;
        if (c >= dv) break;
        for (int rt = 0; rt < kOutRows; ++rt)
            if (rt < RT) store_f(O, (urow + i0 + rt) * dv + c, acc[rt][ci] / den_s[rt]);
    }
}

struct GeneralWs {
    float *MQ, *MK, *Z;
    size_t total;
};

GeneralWs carve(const Problem &pb, void *ws)
{
    GeneralWs w;
    const size_t m_bytes = pb.exact_feat ? 0 : align_up((size_t)pb.units * pb.n * pb.mcols * 4, 256);
    const size_t z_bytes = align_up((size_t)pb.units * pb.t * (size_t)pb.F * (pb.dv + 1) * 4, 256);
    char *base = (char *)ws;
    w.MQ = (float *)base;
    w.MK = (float *)(base + m_bytes);
    w.Z = (float *)(base + 2 * m_bytes);
    w.total = 2 * m_bytes + z_bytes;
    return w;
}

template <typename T>
psf_status sketch_launch(const Problem &pb, const void *X, const void *G, float *M_f32, void *M_out,
                         void *Phi_out, hipStream_t s, const void *X2 = nullptr, float *M2_f32 = nullptr)
{
    const long long rows = (long long)pb.units * pb.n, all = X2 ? 2 * rows : rows;
    const int grid = (int)(all < 65536 ? all : 65536);
    if (pb.learned && pb.p > 2) {
        hipLaunchKernelGGL(gen_sketch_learned_kernel<T>, dim3(grid), dim3(kThreads), 0, s, (const T *)X,
                           (const T *)G, rows, pb.n, pb.heads, pb.per_head ? 1 : 0, pb.d, pb.r, pb.p,
                           pb.g_len, M_f32, (T *)M_out, (T *)Phi_out, (const T *)X2, M2_f32);
        PSF_LAUNCH_CHECK();
        return PSF_OK;
    }
    hipLaunchKernelGGL(gen_sketch_kernel<T>, dim3(grid), dim3(kThreads), 0, s, (const T *)X,
                       (const T *)G, rows, pb.n, pb.heads, pb.per_head ? 1 : 0, pb.d, pb.r, pb.p,
                       pb.exact_feat ? 1 : 0, pb.F, pb.g_len, M_f32, (T *)M_out, (T *)Phi_out, (const T *)X2,
                       M2_f32);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}

template <typename T>
psf_status attn_launch(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                       void *O, void *ws, hipStream_t s, StageTimer *tm, bool noncausal)
{
    GeneralWs w = carve(pb, ws);
    psf_status st;
    if (!pb.exact_feat) {
        st = sketch_launch<T>(pb, Q, G, w.MQ, nullptr, nullptr, s);
        if (st != PSF_OK) return st;
    }
    if (tm) tm->mark();
    if (!pb.exact_feat) {
        st = sketch_launch<T>(pb, K, G, w.MK, nullptr, nullptr, s);
        if (st != PSF_OK) return st;
    }
    if (tm) tm->mark();
    if (pb.t > 1 || noncausal) {                        // H_l of every block but the last; all of them without a mask
        dim3 grid((unsigned)((pb.F + kStateFeat - 1) / kStateFeat), (unsigned)(noncausal ? pb.t : pb.t - 1),
                  (unsigned)pb.units);
        hipLaunchKernelGGL(gen_state_kernel<T>, grid, dim3(kThreads), 0, s, w.MK, (const T *)K,
                           (const T *)V, w.Z, pb.n, pb.d, pb.dv, pb.p, pb.b, pb.t, pb.mcols, pb.F,
                           pb.exact_feat ? 1 : 0);
        PSF_LAUNCH_CHECK();
    }
    if (tm) tm->mark();
    if (pb.t > 1 || noncausal) {
        const size_t per_block = (size_t)pb.F * (pb.dv + 1);
        const size_t total = (size_t)pb.units * per_block;
        const dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
        if (noncausal)
            hipLaunchKernelGGL(gen_total_kernel, grid, dim3(kThreads), 0, s, w.Z, pb.units, pb.t, per_block);
        else
            hipLaunchKernelGGL(gen_scan_kernel, grid, dim3(kThreads), 0, s, w.Z, pb.units, pb.t, per_block);
        PSF_LAUNCH_CHECK();
    }
    if (tm) tm->mark();
    int rows_per_wg = kOutRows;
    while (pb.b % rows_per_wg != 0) rows_per_wg /= 2;
    dim3 grid((unsigned)(pb.n / rows_per_wg), (unsigned)pb.units);
    hipLaunchKernelGGL(gen_out_kernel<T>, grid, dim3(kThreads), 0, s, w.MQ, w.MK, (const T *)Q,
                       (const T *)K, (const T *)V, w.Z, (T *)O, pb.n, pb.d, pb.dv, pb.p, pb.b, pb.t,
                       pb.mcols, pb.F, pb.exact_feat ? 1 : 0, pb.local_exact ? 1 : 0, rows_per_wg,
                       noncausal ? 1 : 0);
    PSF_LAUNCH_CHECK();
    if (tm) tm->mark();
    return PSF_OK;
}

}  // namespace

size_t general_workspace_bytes(const Problem &pb)
{
    return carve(pb, nullptr).total;
}

psf_status general_sketch(const Problem &pb, const void *X, const void *G, void *M_out, void *Phi_out,
                          hipStream_t s)
{
    if (pb.exact_feat && !Phi_out) return PSF_ERR_NULL;   // exact features have no m(x)
    return pb.bf16 ? sketch_launch<bf16_t>(pb, X, G, nullptr, M_out, Phi_out, s)
                   : sketch_launch<float>(pb, X, G, nullptr, M_out, Phi_out, s);
}

psf_status general_sketch_f32(const Problem &pb, const void *X, const void *G, float *M_f32, hipStream_t s)
{
    return pb.bf16 ? sketch_launch<bf16_t>(pb, X, G, M_f32, nullptr, nullptr, s)
                   : sketch_launch<float>(pb, X, G, M_f32, nullptr, nullptr, s);
}

psf_status general_sketch_pair_f32(const Problem &pb, const void *X, const void *X2, const void *G, float *M_f32,
                                   float *M2_f32, hipStream_t s)
{
    return pb.bf16 ? sketch_launch<bf16_t>(pb, X, G, M_f32, nullptr, nullptr, s, X2, M2_f32)
                   : sketch_launch<float>(pb, X, G, M_f32, nullptr, nullptr, s, X2, M2_f32);
}

psf_status general_attn(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                        void *O, void *ws, hipStream_t s, StageTimer *tm, bool noncausal)
{
    return pb.bf16 ? attn_launch<bf16_t>(pb, Q, K, V, G, O, ws, s, tm, noncausal)
                   : attn_launch<float>(pb, Q, K, V, G, O, ws, s, tm, noncausal);
}

}  // namespace psf
