// Backward pass of causal Polysketch attention (PolySketchFormer, arXiv 2310.01655): gradient
// of the function of Section 3 (weights of Sections 3.1 / 3.2, sketch of Algorithm 1) with
// respect to Q, K, V, evaluated with the same block decomposition as the forward pass.
//
// With C_j = [v_j | 1], phi_i = phi'(q_i), psi_j = phi'(k_j), H_l = sum_{j in block l} psi_j C_j^T,
// Z_l = sum_{l' < l} H_l' (Section 3.1) and row_i = [N_i | S_i] = phi_i^T Z_l + (in-block term):
//   D_i = 1 + S_i,  o_i = N_i / D_i,  G_i = [dO_i / D_i | -<dO_i, o_i> / D_i],
//   dL/dw_ij = <G_i, C_j>                                      for every pair j <= i,
//   pairs in different blocks (w_ij = <phi_i, psi_j>):
//     dphi_i = Z_l G_i,   dpsi_j = R_l C_j,   dC_j = R_l^T psi_j,
//     R_l = sum_{l' > l} sum_{i in block l'} phi_i G_i^T      (the mirror image of Z_l),
//     and phi = m (x) m gives dm[a] = sum_b (dphi[a,b] + dphi[b,a]) m[b];
//   pairs inside a block: w = <q,k>^p (Section 3.2) or <m(q),m(k)>^2 (Section 3.1), pair by pair;
//   finally dQ += J^T dm(Q), dK += J^T dm(K) through Algorithm 1.
// These are plain fp32 LDS-staged kernels for every descriptor with sketch features (any d, dv,
// r <= 256, p in {2,4,8,16}, either in-block rule, fp32 or bf16 storage).  The sketch matrices
// are constants.  With learned sketches (Algorithm 2) the last step goes through the networks
// instead and can also return the gradient with respect to their parameters.
#include "psf_internal.h"

namespace psf {
namespace {

constexpr int kThreads = 256;
constexpr int kRows = 8;            // tokens per workgroup in the row / column kernels (at most)
constexpr int kChunk = 256;         // features or tokens staged per step and row (8 KB of LDS for 8 rows)
constexpr int kStateFeat = 32;     // features per workgroup in the state kernel
constexpr int kStateChunk = 64;    // tokens staged per step in the state kernel

__device__ __forceinline__ float pow_int(float x, int p)
{
    float y = 1.f;
    for (int e = 0; e < p; ++e) y *= x;
    return y;
}

// C[row] = [v_row | 1]
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_cv_kernel(const T *__restrict__ V, float *__restrict__ CV,
                                                          size_t rows, int dv)
{
    const int kc = dv + 1;
    const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= rows * kc) return;
    const size_t row = idx / kc;
    const int c = (int)(idx % kc);
    CV[idx] = c < dv ? load_f(V, row * dv + c) : 1.f;
}

// H[u][l][f][c] = sum_{j in block l} M[j][f / mcols] M[j][f % mcols] C[j][c]
__global__ __launch_bounds__(kThreads) void bwd_state_kernel(const float *__restrict__ M,
                                                             const float *__restrict__ C,
                                                             float *__restrict__ H, int n, int kc, int b,
                                                             int t, int mcols, long long F)
{
    __shared__ float phi[kStateChunk][kStateFeat];
    const int tid = threadIdx.x, l = blockIdx.y, u = blockIdx.z;
    const long long f0 = (long long)blockIdx.x * kStateFeat;
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
                v = M[row * mcols + f / mcols] * M[row * mcols + f % mcols];
            }
            phi[jj][ff] = v;
        }
        __syncthreads();
        const int lim = min(kStateChunk, b - j0);
        for (int ci = 0; ci < 2; ++ci) {
            const int c = tid + ci * kThreads;
            if (c >= kc) break;
            for (int jj = 0; jj < lim; ++jj) {
                const float v = C[(row0 + j0 + jj) * kc + c];
                for (int ff = 0; ff < kStateFeat; ++ff) acc[ff][ci] += phi[jj][ff] * v;
            }
        }
    }
    float *h = H + (((size_t)u * t + l) * (size_t)F) * kc;
    for (int ci = 0; ci < 2; ++ci) {
        const int c = tid + ci * kThreads;
        if (c >= kc) break;
        for (int ff = 0; ff < kStateFeat; ++ff)
            if (f0 + ff < F) h[(size_t)(f0 + ff) * kc + c] = acc[ff][ci];
    }
}

// In place: exclusive prefix over blocks (reverse == 0: Z_l = sum_{l' < l} H_l') or exclusive
// suffix (reverse != 0: R_l = sum_{l' > l} H_l'), sequential as in Section 3.1.
__global__ __launch_bounds__(kThreads) void bwd_scan_kernel(float *__restrict__ Z, int units, int t,
                                                            size_t per_block, int reverse)
{
    const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= (size_t)units * per_block) return;
    const size_t u = idx / per_block, e = idx % per_block;
    float *z = Z + u * (size_t)t * per_block + e;
    float run = 0.f;
    for (int s = 0; s < t; ++s) {
        const int l = reverse ? t - 1 - s : s;
        const float h = z[(size_t)l * per_block];
        z[(size_t)l * per_block] = run;
        run += h;
    }
}

// ---- helpers for one workgroup of RT rows (RT <= kRows) ------------------------------------
// Every workgroup handles RT consecutive tokens of one block, so that a state (F x kc floats)
// is streamed once per RT tokens.  LDS arrays are [kRows][pitch].

// out[rt][c] += sum_{k < K} wt[k][rt] * Mat[k * ld + c] for c < kc; wt ([K][kRows], rows
// rt >= RT hold zeros) and out in LDS.  The threads are split into slices over k; `red` is
// kRows * kThreads floats of LDS scratch.  Reads of Mat are contiguous in c.
__device__ void wg_weighted_rows(const float *wt, int RT, int K, const float *__restrict__ Mat,
                                 size_t ld, int kc, float *out, int out_pitch, float *red)
{
    const int tid = threadIdx.x;
    int kcp = 32;
    while (kcp < kc && kcp < kThreads) kcp *= 2;        // columns per slice (power of two)
    const int nsl = kThreads / kcp;
    for (int c0 = 0; c0 < kc; c0 += kcp) {
        const int c = c0 + tid % kcp, sl = tid / kcp;
        float a[kRows];
        for (int rt = 0; rt < kRows; ++rt) a[rt] = 0.f;
        if (c < kc)
            for (int k = sl; k < K; k += nsl) {
                const float mv = Mat[(size_t)k * ld + c];
                const float4 w0 = *(const float4 *)&wt[k * kRows], w1 = *(const float4 *)&wt[k * kRows + 4];
                a[0] += w0.x * mv; a[1] += w0.y * mv; a[2] += w0.z * mv; a[3] += w0.w * mv;
                a[4] += w1.x * mv; a[5] += w1.y * mv; a[6] += w1.z * mv; a[7] += w1.w * mv;
            }
        __syncthreads();
        for (int rt = 0; rt < kRows; ++rt) red[rt * kThreads + tid] = a[rt];
        __syncthreads();
        for (int idx = tid; idx < RT * kcp; idx += kThreads) {
            const int rt = idx / kcp, cc = idx % kcp;
            if (c0 + cc < kc) {
                float sacc = 0.f;
                for (int q = 0; q < nsl; ++q) sacc += red[rt * kThreads + q * kcp + cc];
                out[rt * out_pitch + c0 + cc] += sacc;
            }
        }
        __syncthreads();
    }
}

// dm[rt][a] += 2 sum_c g[rt][c] sum_b mT[b][rt] S[(a * mcols + b) * kc + c]: the contraction of
// a state S (mcols^2 features x kc columns, symmetric in its two sketch indices because
// phi' = m (x) m) with g over the columns and with m over one sketch index; by that symmetry
// this equals sum_b (T[a,b] + T[b,a]) m[b] for T = S g.  mT is [mcols][kRows] (rows rt >= RT
// zero), g is [kRows][g_pitch], dm [kRows][dm_pitch]; wsum is 4 * kRows floats of LDS.  Thread (c, slice) walks the
// rows a of its slice, so reads of S are contiguous in c and every dm entry has one writer.
__device__ void wg_state_bilinear(const float *__restrict__ S, int kc, int mcols, int RT,
                                  const float *mT, const float *g, int g_pitch, float *dm,
                                  int dm_pitch, float *wsum)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int kcp = 32;
    while (kcp < kc && kcp < kThreads) kcp *= 2;
    const int nsl = kThreads / kcp, c = tid % kcp, sl = tid / kcp;
    const int iters = (mcols + nsl - 1) / nsl;
    for (int c0 = 0; c0 < kc; c0 += kcp) {                  // one pass unless kc = 257
        const int cc = c0 + c;
        for (int it = 0; it < iters; ++it) {
            const int a = it * nsl + sl;
            float part[kRows];
            for (int rt = 0; rt < kRows; ++rt) part[rt] = 0.f;
            if (a < mcols && cc < kc) {
                const float *sa = S + (size_t)a * mcols * kc + cc;
                for (int bq = 0; bq < mcols; ++bq) {
                    const float zv = sa[(size_t)bq * kc];
                    const float4 m0 = *(const float4 *)&mT[bq * kRows], m1 = *(const float4 *)&mT[bq * kRows + 4];
                    part[0] += m0.x * zv; part[1] += m0.y * zv; part[2] += m0.z * zv; part[3] += m0.w * zv;
                    part[4] += m1.x * zv; part[5] += m1.y * zv; part[6] += m1.z * zv; part[7] += m1.w * zv;
                }
                for (int rt = 0; rt < kRows; ++rt) part[rt] *= (rt < RT) ? g[rt * g_pitch + cc] : 0.f;
            }
            const int width = kcp < 64 ? kcp : 64;          // lanes of this slice inside the wave
            for (int off = width / 2; off > 0; off >>= 1)
                for (int rt = 0; rt < kRows; ++rt) part[rt] += __shfl_xor(part[rt], off);
            if (kcp <= 64) {
                if (lane % kcp == 0 && a < mcols)
                    for (int rt = 0; rt < kRows; ++rt)
                        if (rt < RT) dm[rt * dm_pitch + a] += 2.f * part[rt];
            } else {
                const int wps = kcp / 64;                   // waves per slice
                __syncthreads();
                if (lane == 0)
                    for (int rt = 0; rt < kRows; ++rt) wsum[wave * kRows + rt] = part[rt];
                __syncthreads();
                if (c == 0 && a < mcols)
                    for (int rt = 0; rt < kRows; ++rt)
                        if (rt < RT) {
                            float sacc = 0.f;
                            for (int w = 0; w < wps; ++w) sacc += wsum[(sl * wps + w) * kRows + rt];
                            dm[rt * dm_pitch + a] += 2.f * sacc;
                        }
            }
        }
    }
    __syncthreads();
}

// LDS of the three token kernels is carved at run time from the actual sizes (d, dv, sketch
// columns), so that the common shapes keep several workgroups per CU.  In-block pairs are
// handled tile by tile: kTile tokens of the other side are staged in LDS (rows padded by one
// float) together with their [V | 1] or G rows, then every (token, staged token) pair is one
// thread's dot product out of LDS.
constexpr int kTile = 32;

struct Carver {
    float *base;
    size_t used = 0;
    __host__ __device__ explicit Carver(float *b) : base(b) {}
    __host__ __device__ float *take(size_t floats)
    {
        float *p = base + used;
        used += (floats + 3) & ~(size_t)3;              // keep 16-byte alignment
        return p;
    }
};

// rows [r0, r0 + nr) of a row-major array of `width` columns -> LDS tile with pitch width + 1
template <typename S>
__device__ __forceinline__ void stage_rows(const S *__restrict__ src, size_t r0, int nr, int width,
                                           float *dst)
{
    for (int idx = threadIdx.x; idx < nr * width; idx += kThreads)
        dst[(idx / width) * (width + 1) + idx % width] = load_f(src, r0 * width + idx);
}

struct TokenLds {                                        // what every token kernel carves
    float *wt, *red, *mT, *wsum, *ta, *tc, *pw, *pd;
};
__host__ __device__ inline size_t carve_common(Carver &cv, TokenLds *t, int wa, int kc, int mcols)
{
    TokenLds x;
    x.wt = cv.take((size_t)kRows * kChunk);              // features of RT tokens, [k][kRows]
    x.red = cv.take((size_t)kRows * kThreads);
    x.mT = cv.take((size_t)mcols * kRows);
    x.wsum = cv.take(4 * kRows);
    x.ta = cv.take((size_t)kTile * (wa + 1));            // staged q / k (or m) rows
    x.tc = cv.take((size_t)kTile * (kc + 1));            // staged [V | 1] or G rows
    x.pw = cv.take((size_t)kRows * kTile);               // pair weights
    x.pd = cv.take((size_t)kRows * kTile);               // pair gradients
    if (t) *t = x;
    return cv.used;
}

// ---- forward rows and G_i ------------------------------------------------------------
// Rows i0 .. i0 + RT - 1 of one block: row_i = phi_i^T Z_l + sum_{j <= i, same block} w_ij C_j,
// then GC[i] = [dO_i / D_i | -<dO_i, o_i> / D_i].
__host__ __device__ inline size_t rows_lds(float *base, int d, int kc, int mcols, int wa, TokenLds *t,
                                           float **rowv, float **mq, float **qs, float **dots)
{
    Carver cv(base);
    carve_common(cv, t, wa, kc, mcols);
    float *a = cv.take((size_t)kRows * kc), *b2 = cv.take((size_t)kRows * mcols),
          *c = cv.take((size_t)kRows * d), *e = cv.take(2 * kRows);
    if (rowv) { *rowv = a; *mq = b2; *qs = c; *dots = e; }
    return cv.used * sizeof(float);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_rows_kernel(
    const float *__restrict__ MQ, const float *__restrict__ MK, const T *__restrict__ Q,
    const T *__restrict__ K, const float *__restrict__ CV, const float *__restrict__ Z,
    const T *__restrict__ dO, float *__restrict__ GC, int n, int d, int dv, int p, int b, int t,
    int mcols, long long F, int local_exact, int RT)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int tid = threadIdx.x, i0 = blockIdx.x * RT, u = blockIdx.y;
    const int l = i0 / b, kc = dv + 1, wa = local_exact ? d : mcols;
    TokenLds L;
    float *rowv, *mq, *qs, *dots;
    rows_lds(smem, d, kc, mcols, wa, &L, &rowv, &mq, &qs, &dots);
    const size_t urow = (size_t)u * n;
    for (int idx = tid; idx < kRows * kChunk; idx += kThreads) L.wt[idx] = 0.f;   // rows >= RT stay zero
    for (int idx = tid; idx < RT * kc; idx += kThreads) rowv[idx] = 0.f;
    for (int idx = tid; idx < RT * mcols; idx += kThreads) mq[idx] = MQ[(urow + i0) * mcols + idx];
    for (int idx = tid; idx < RT * d; idx += kThreads) qs[idx] = load_f(Q, (urow + i0) * d + idx);
    __syncthreads();
    if (l > 0) {
        const float *z = Z + (((size_t)u * t + l) * (size_t)F) * kc;
        for (long long f0 = 0; f0 < F; f0 += kChunk) {
            const int nf = (int)min((long long)kChunk, F - f0);
            __syncthreads();
            for (int idx = tid; idx < RT * nf; idx += kThreads) {
                const int rt = idx / nf, ff = idx % nf;
                const long long f = f0 + ff;
                L.wt[ff * kRows + rt] = mq[rt * mcols + f / mcols] * mq[rt * mcols + f % mcols];
            }
            __syncthreads();
            wg_weighted_rows(L.wt, RT, nf, z + (size_t)f0 * kc, kc, kc, rowv, kc, L.red);
        }
    }
    const float *qrow = local_exact ? qs : mq;
    const int jbeg = l * b, jend = i0 + RT;               // keys jbeg .. jend - 1; row rt keeps j <= i0 + rt
    for (int j0 = jbeg; j0 < jend; j0 += kTile) {
        const int nj = min(kTile, jend - j0);
        __syncthreads();
        if (local_exact) stage_rows(K, urow + j0, nj, d, L.ta);
        else stage_rows(MK, urow + j0, nj, mcols, L.ta);
        stage_rows(CV, urow + j0, nj, kc, L.tc);
        __syncthreads();
        for (int idx = tid; idx < RT * nj; idx += kThreads) {
            const int rt = idx / nj, jj = idx % nj;
            float w = 0.f;
            if (j0 + jj <= i0 + rt) {
                float sdot = 0.f;
                for (int e = 0; e < wa; ++e) sdot += qrow[rt * wa + e] * L.ta[jj * (wa + 1) + e];
                w = local_exact ? pow_int(sdot, p) : sdot * sdot;
            }
            L.pw[rt * kTile + jj] = w;
        }
        __syncthreads();
        for (int idx = tid; idx < RT * kc; idx += kThreads) {
            const int rt = idx / kc, c = idx % kc;
            float a = 0.f;
            for (int jj = 0; jj < nj; ++jj) a += L.pw[rt * kTile + jj] * L.tc[jj * (kc + 1) + c];
            rowv[rt * kc + c] += a;
        }
    }
    __syncthreads();
    if (tid < RT) {                                       // <dO_i, N_i>, D_i
        const size_t row = urow + i0 + tid;
        float sdot = 0.f;
        for (int c = 0; c < dv; ++c) sdot += load_f(dO, row * dv + c) * rowv[tid * kc + c];
        const float den = 1.f + rowv[tid * kc + dv];
        dots[2 * tid] = den;
        dots[2 * tid + 1] = -(sdot / den) / den;          // -<dO_i, o_i> / D_i
    }
    __syncthreads();
    for (int idx = tid; idx < RT * dv; idx += kThreads) {
        const int rt = idx / dv, c = idx % dv;
        const size_t row = urow + i0 + rt;
        GC[row * kc + c] = load_f(dO, row * dv + c) / dots[2 * rt];
    }
    if (tid < RT) GC[(urow + i0 + tid) * kc + dv] = dots[2 * tid + 1];
}

// ---- gradient with respect to the query side, rows i0 .. i0 + RT - 1 ---------------------
__host__ __device__ inline size_t q_lds(float *base, int d, int kc, int mcols, int wa, TokenLds *t,
                                        float **g, float **mq, float **qs, float **dm, float **dq)
{
    Carver cv(base);
    carve_common(cv, t, wa, kc, mcols);
    float *a = cv.take((size_t)kRows * kc), *b2 = cv.take((size_t)kRows * mcols),
          *c = cv.take((size_t)kRows * d), *e = cv.take((size_t)kRows * mcols),
          *f = cv.take((size_t)kRows * d);
    if (g) { *g = a; *mq = b2; *qs = c; *dm = e; *dq = f; }
    return cv.used * sizeof(float);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_q_kernel(
    const float *__restrict__ MQ, const float *__restrict__ MK, const T *__restrict__ Q,
    const T *__restrict__ K, const float *__restrict__ CV, const float *__restrict__ GC,
    const float *__restrict__ Z, float *__restrict__ dMQ, float *__restrict__ dQd, int n, int d,
    int dv, int p, int b, int t, int mcols, long long F, int local_exact, int RT)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int tid = threadIdx.x, i0 = blockIdx.x * RT, u = blockIdx.y;
    const int l = i0 / b, kc = dv + 1, wa = local_exact ? d : mcols;
    TokenLds L;
    float *g, *mq, *qs, *dm, *dq;
    q_lds(smem, d, kc, mcols, wa, &L, &g, &mq, &qs, &dm, &dq);
    const size_t urow = (size_t)u * n;
    for (int idx = tid; idx < RT * kc; idx += kThreads) g[idx] = GC[(urow + i0) * kc + idx];
    for (int idx = tid; idx < kRows * mcols; idx += kThreads) {
        const int rt = idx / mcols, e = idx % mcols;
        const float mv = rt < RT ? MQ[(urow + i0 + rt) * mcols + e] : 0.f;
        mq[idx] = mv;
        L.mT[e * kRows + rt] = mv;
        dm[idx] = 0.f;
    }
    for (int idx = tid; idx < RT * d; idx += kThreads) {
        qs[idx] = load_f(Q, (urow + i0) * d + idx);
        dq[idx] = 0.f;
    }
    __syncthreads();
    if (l > 0) {
        const float *z = Z + (((size_t)u * t + l) * (size_t)F) * kc;
        wg_state_bilinear(z, kc, mcols, RT, L.mT, g, kc, dm, mcols, L.wsum);
    }
    __syncthreads();
    const float *qrow = local_exact ? qs : mq;
    float *gout = local_exact ? dq : dm;                  // where the in-block term goes
    const int jbeg = l * b, jend = i0 + RT;
    for (int j0 = jbeg; j0 < jend; j0 += kTile) {
        const int nj = min(kTile, jend - j0);
        __syncthreads();
        if (local_exact) stage_rows(K, urow + j0, nj, d, L.ta);
        else stage_rows(MK, urow + j0, nj, mcols, L.ta);
        stage_rows(CV, urow + j0, nj, kc, L.tc);
        __syncthreads();
        for (int idx = tid; idx < RT * nj; idx += kThreads) {
            const int rt = idx / nj, jj = idx % nj;
            float val = 0.f;
            if (j0 + jj <= i0 + rt) {
                float dw = 0.f, sdot = 0.f;
                for (int c = 0; c < kc; ++c) dw += g[rt * kc + c] * L.tc[jj * (kc + 1) + c];
                for (int e = 0; e < wa; ++e) sdot += qrow[rt * wa + e] * L.ta[jj * (wa + 1) + e];
                val = local_exact ? (float)p * pow_int(sdot, p - 1) * dw : 2.f * sdot * dw;
            }
            L.pd[rt * kTile + jj] = val;
        }
        __syncthreads();
        for (int idx = tid; idx < RT * wa; idx += kThreads) {
            const int rt = idx / wa, e = idx % wa;
            float a = 0.f;
            for (int jj = 0; jj < nj; ++jj) a += L.pd[rt * kTile + jj] * L.ta[jj * (wa + 1) + e];
            gout[rt * wa + e] += a;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < RT * mcols; idx += kThreads) dMQ[(urow + i0) * mcols + idx] = dm[idx];
    for (int idx = tid; idx < RT * d; idx += kThreads) dQd[(urow + i0) * d + idx] = dq[idx];
}

// ---- gradient with respect to the key side and V, columns j0 .. j0 + RT - 1 ----------------
__host__ __device__ inline size_t k_lds(float *base, int d, int kc, int mcols, int wa, TokenLds *t,
                                        float **cj, float **dc, float **mk, float **ks, float **dm,
                                        float **dk)
{
    Carver cv(base);
    carve_common(cv, t, wa, kc, mcols);
    float *a = cv.take((size_t)kRows * kc), *b2 = cv.take((size_t)kRows * kc),
          *c = cv.take((size_t)kRows * mcols), *e = cv.take((size_t)kRows * d),
          *f = cv.take((size_t)kRows * mcols), *h = cv.take((size_t)kRows * d);
    if (cj) { *cj = a; *dc = b2; *mk = c; *ks = e; *dm = f; *dk = h; }
    return cv.used * sizeof(float);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_k_kernel(
    const float *__restrict__ MQ, const float *__restrict__ MK, const T *__restrict__ Q,
    const T *__restrict__ K, const float *__restrict__ CV, const float *__restrict__ GC,
    const float *__restrict__ RB, float *__restrict__ dMK, float *__restrict__ dKd,
    T *__restrict__ dV, int n, int d, int dv, int p, int b, int t, int mcols, long long F,
    int local_exact, int RT)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int tid = threadIdx.x, j0 = blockIdx.x * RT, u = blockIdx.y;
    const int l = j0 / b, kc = dv + 1, wa = local_exact ? d : mcols;
    TokenLds L;
    float *cj, *dc, *mk, *ks, *dm, *dk;
    k_lds(smem, d, kc, mcols, wa, &L, &cj, &dc, &mk, &ks, &dm, &dk);
    const size_t urow = (size_t)u * n;
    for (int idx = tid; idx < kRows * kChunk; idx += kThreads) L.wt[idx] = 0.f;   // rows >= RT stay zero
    for (int idx = tid; idx < RT * kc; idx += kThreads) {
        cj[idx] = CV[(urow + j0) * kc + idx];
        dc[idx] = 0.f;
    }
    for (int idx = tid; idx < kRows * mcols; idx += kThreads) {
        const int rt = idx / mcols, e = idx % mcols;
        const float mv = rt < RT ? MK[(urow + j0 + rt) * mcols + e] : 0.f;
        mk[idx] = mv;
        L.mT[e * kRows + rt] = mv;
        dm[idx] = 0.f;
    }
    for (int idx = tid; idx < RT * d; idx += kThreads) {
        ks[idx] = load_f(K, (urow + j0) * d + idx);
        dk[idx] = 0.f;
    }
    __syncthreads();
    if (l < t - 1) {
        const float *rb = RB + (((size_t)u * t + l) * (size_t)F) * kc;
        wg_state_bilinear(rb, kc, mcols, RT, L.mT, cj, kc, dm, mcols, L.wsum);
        for (long long f0 = 0; f0 < F; f0 += kChunk) {            // dC_j = R_l^T psi_j
            const int nf = (int)min((long long)kChunk, F - f0);
            __syncthreads();
            for (int idx = tid; idx < RT * nf; idx += kThreads) {
                const int rt = idx / nf, ff = idx % nf;
                const long long f = f0 + ff;
                L.wt[ff * kRows + rt] = mk[rt * mcols + f / mcols] * mk[rt * mcols + f % mcols];
            }
            __syncthreads();
            wg_weighted_rows(L.wt, RT, nf, rb + (size_t)f0 * kc, kc, kc, dc, kc, L.red);
        }
    }
    __syncthreads();
    // in-block pairs: rows i = j0 .. iend - 1; column rt keeps i >= j0 + rt
    const float *krow = local_exact ? ks : mk;
    float *gout = local_exact ? dk : dm;
    const int iend = (l + 1) * b;
    for (int ib = j0; ib < iend; ib += kTile) {
        const int ni = min(kTile, iend - ib);
        __syncthreads();
        if (local_exact) stage_rows(Q, urow + ib, ni, d, L.ta);
        else stage_rows(MQ, urow + ib, ni, mcols, L.ta);
        stage_rows(GC, urow + ib, ni, kc, L.tc);
        __syncthreads();
        for (int idx = tid; idx < RT * ni; idx += kThreads) {
            const int rt = idx / ni, ii = idx % ni;
            float w = 0.f, val = 0.f;
            if (ib + ii >= j0 + rt) {
                float dw = 0.f, sdot = 0.f;
                for (int c = 0; c < kc; ++c) dw += L.tc[ii * (kc + 1) + c] * cj[rt * kc + c];
                for (int e = 0; e < wa; ++e) sdot += L.ta[ii * (wa + 1) + e] * krow[rt * wa + e];
                w = local_exact ? pow_int(sdot, p) : sdot * sdot;
                val = local_exact ? (float)p * pow_int(sdot, p - 1) * dw : 2.f * sdot * dw;
            }
            L.pw[rt * kTile + ii] = w;
            L.pd[rt * kTile + ii] = val;
        }
        __syncthreads();
        for (int idx = tid; idx < RT * wa; idx += kThreads) {
            const int rt = idx / wa, e = idx % wa;
            float a = 0.f;
            for (int ii = 0; ii < ni; ++ii) a += L.pd[rt * kTile + ii] * L.ta[ii * (wa + 1) + e];
            gout[rt * wa + e] += a;
        }
        for (int idx = tid; idx < RT * dv; idx += kThreads) {     // dV_j += sum_i w_ij g_i
            const int rt = idx / dv, c = idx % dv;
            float a = 0.f;
            for (int ii = 0; ii < ni; ++ii) a += L.pw[rt * kTile + ii] * L.tc[ii * (kc + 1) + c];
            dc[rt * kc + c] += a;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < RT * mcols; idx += kThreads) dMK[(urow + j0) * mcols + idx] = dm[idx];
    for (int idx = tid; idx < RT * d; idx += kThreads) dKd[(urow + j0) * d + idx] = dk[idx];
    for (int idx = tid; idx < RT * dv; idx += kThreads)
        store_f(dV, (urow + j0 + idx / dv) * dv + idx % dv, dc[(idx / dv) * kc + idx % dv]);
}

// ---- gradient through Algorithm 1, one row per loop iteration --------------------------
// Recomputes the recursion level by level (as the forward sketch kernel does), keeping the two
// projections U, W of every node, then walks back: dU = sqrt(1/r) dM * W, dW = sqrt(1/r) dM * U,
// dM(child 1) = dU G1^T, dM(child 2) = dW G2^T.  dX = that + the direct term.
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_sketch_kernel(
    const T *__restrict__ X, const T *__restrict__ G, const float *__restrict__ dM,
    const float *__restrict__ direct, T *__restrict__ dX, long long rows, int n, int heads,
    int per_head, int d, int r, int p, size_t g_len)
{
    constexpr int kNodes = 7;                                  // p <= 16: 4 + 2 + 1 nodes
    __shared__ float xs[PSF_MAX_DIM], dx[PSF_MAX_DIM];
    __shared__ float U[kNodes][PSF_MAX_DIM], W[kNodes][PSF_MAX_DIM], Mv[kNodes][PSF_MAX_DIM],
        dMv[kNodes][PSF_MAX_DIM];
    const int tid = threadIdx.x;
    for (long long row = blockIdx.x; row < rows; row += gridDim.x) {
        __syncthreads();
        if (tid < d) { xs[tid] = load_f(X, (size_t)row * d + tid); dx[tid] = direct[(size_t)row * d + tid]; }
        __syncthreads();
        if (p == 2) {
            if (tid < d) store_f(dX, (size_t)row * d + tid, dx[tid] + dM[(size_t)row * d + tid]);
            continue;
        }
        const int head = (int)((row / n) % heads);
        const T *g_first = G + (per_head ? (size_t)head * g_len : 0);
        const T *g_inner = g_first + (size_t)(p / 2) * d * r;
        const float sc = sqrtf(1.0f / (float)r);
        // forward: level 0 nodes 0 .. p/4 - 1, next level after them, ...
        int count = p / 4, first = 0;
        if (tid < r) {
            for (int j = 0; j < count; ++j) {
                const T *ga = g_first + (size_t)(2 * j) * d * r, *gb = ga + (size_t)d * r;
                float a = 0.f, w = 0.f;
                for (int e = 0; e < d; ++e) {
                    a += xs[e] * load_f(ga, (size_t)e * r + tid);
                    w += xs[e] * load_f(gb, (size_t)e * r + tid);
                }
                U[j][tid] = a; W[j][tid] = w; Mv[j][tid] = sc * (a * w);
            }
        }
        __syncthreads();
        size_t inner_at = 0;
        while (count > 1) {
            const int next = count / 2, base = first + count;
            if (tid < r) {
                for (int j = 0; j < next; ++j) {
                    const T *ga = g_inner + (inner_at + 2 * j) * (size_t)r * r, *gb = ga + (size_t)r * r;
                    const float *m1 = Mv[first + 2 * j], *m2 = Mv[first + 2 * j + 1];
                    float a = 0.f, w = 0.f;
                    for (int e = 0; e < r; ++e) {
                        a += m1[e] * load_f(ga, (size_t)e * r + tid);
                        w += m2[e] * load_f(gb, (size_t)e * r + tid);
                    }
                    U[base + j][tid] = a; W[base + j][tid] = w; Mv[base + j][tid] = sc * (a * w);
                }
            }
            __syncthreads();
            inner_at += 2 * (size_t)next;
            first = base;
            count = next;
        }
        // backward: `first` is the root now
        if (tid < r) dMv[first][tid] = dM[(size_t)row * r + tid];
        __syncthreads();
        while (true) {
            // turn dM of the nodes of this level into dU, dW (in place of U, W)
            if (tid < r) {
                for (int j = 0; j < count; ++j) {
                    const float gm = sc * dMv[first + j][tid];
                    const float a = U[first + j][tid], w = W[first + j][tid];
                    U[first + j][tid] = gm * w;
                    W[first + j][tid] = gm * a;
                }
            }
            __syncthreads();
            if (first == 0) break;
            const int below = count * 2, bfirst = first - below;
            inner_at -= 2 * (size_t)count;
            if (tid < r) {
                for (int j = 0; j < count; ++j) {
                    const T *ga = g_inner + (inner_at + 2 * j) * (size_t)r * r, *gb = ga + (size_t)r * r;
                    float a = 0.f, w = 0.f;
                    for (int c = 0; c < r; ++c) {
                        a += U[first + j][c] * load_f(ga, (size_t)tid * r + c);
                        w += W[first + j][c] * load_f(gb, (size_t)tid * r + c);
                    }
                    dMv[bfirst + 2 * j][tid] = a;
                    dMv[bfirst + 2 * j + 1][tid] = w;
                }
            }
            __syncthreads();
            first = bfirst;
            count = below;
        }
        if (tid < d) {
            float a = dx[tid];
            for (int j = 0; j < p / 4; ++j) {
                const T *ga = g_first + (size_t)(2 * j) * d * r, *gb = ga + (size_t)d * r;
                for (int c = 0; c < r; ++c)
                    a += U[j][c] * load_f(ga, (size_t)tid * r + c) + W[j][c] * load_f(gb, (size_t)tid * r + c);
            }
            store_f(dX, (size_t)row * d + tid, a);
        }
    }
}

// ---- gradient through Algorithm 2 (learned sketches, Appendix D) ---------------------------
// One network is LN -> W1 (win x 8r) -> gelu -> LN -> W2 (8r x r) -> W3 (r x 8r) -> gelu -> W4 (8r x r)
// (the reading stated in include/psf.h); a node returns sqrt(r) tanh(f1(M1) * f2(M2) / sqrt(r)).
// A workgroup takes one row: it runs the networks forward (twice: once for the values every node
// needs, once more per network for the quantities its reverse pass reads), walks back from the
// root, and leaves, per network, the input and the output gradient of every dense layer (and
// the two products a layer normalisation's scale and bias need) in a staging buffer; the
// parameter gradients are then sums over rows of outer products of those, formed by
// bwd_param_gemm / bwd_param_colsum in a fixed order (chunk by chunk, rows in order: no atomics).
constexpr int kMaxHidden = 8 * PSF_MAX_DIM;

__device__ __forceinline__ float gelu_tanh_f(float x)
{
    return 0.5f * x * (1.0f + tanhf(0.7978845608028654f * (x + 0.044715f * x * x * x)));
}

__device__ __forceinline__ float gelu_tanh_grad_f(float x)
{
    const float c = 0.7978845608028654f, k = 0.044715f;
    const float th = tanhf(c * (x + k * x * x * x));
    return 0.5f * (1.0f + th) + 0.5f * x * (1.0f - th * th) * c * (1.0f + 3.0f * k * x * x);
}

// sum of v over the workgroup, the same value in every thread; red: 4 floats of LDS
__device__ __forceinline__ float wg_sum(float v, float *red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// Staging of one network for a chunk of RC rows: offsets (in floats) of its arrays, each [RC][width].
struct NetStage {
    size_t A1, LG1, LB1;                 // width win: layer-norm-1 output; d(out) * xhat; d(out)
    size_t D1, A2, LG2, LB2, D3, A4;     // width 8r: d(pre-gelu 1); LN-2 output; its two products; d(pre-gelu 3); gelu 3
    size_t D2, A3, D4;                   // width r: d(W2 output); W2 output; d(network output)
    size_t end;
};

__host__ __device__ inline NetStage net_stage(size_t base, size_t RC, int win, int r)
{
    const size_t hid = 8 * (size_t)r;
    NetStage L;
    size_t o = base;
    L.A1 = o; o += RC * win;
    L.LG1 = o; o += RC * win;
    L.LB1 = o; o += RC * win;
    L.D1 = o; o += RC * hid;
    L.A2 = o; o += RC * hid;
    L.LG2 = o; o += RC * hid;
    L.LB2 = o; o += RC * hid;
    L.D3 = o; o += RC * hid;
    L.A4 = o; o += RC * hid;
    L.D2 = o; o += RC * r;
    L.A3 = o; o += RC * r;
    L.D4 = o; o += RC * r;
    L.end = o;
    return L;
}

__host__ __device__ inline size_t learned_net_len(int win, int r)
{
    const size_t hid = 8 * (size_t)r;
    return 2 * (size_t)win + (size_t)win * hid + 2 * hid + hid * r + (size_t)r * hid + hid * r;
}

// input width of network k (Appendix D order: the p/2 networks on x, then the ones on sketches)
__host__ __device__ inline int learned_net_win(int k, int d, int r, int p) { return k < p / 2 ? d : r; }

struct LearnedLds {
    float a1[kMaxHidden], xh2[kMaxHidden], a3[kMaxHidden], s1[kMaxHidden];
    float xh1[PSF_MAX_DIM], u[PSF_MAX_DIM], u2[PSF_MAX_DIM], du2[PSF_MAX_DIM], tw[PSF_MAX_DIM];
    float red[4];
};

// out[c] = sum_e x[e] W[e * cols + c]; x, out in LDS
template <typename T>
__device__ void wgl_dense(const float *x, int rows, const T *W, int cols, float *out)
{
    for (int c = threadIdx.x; c < cols; c += kThreads) {
        float a = 0.f;
        for (int e = 0; e < rows; ++e) a += x[e] * load_f(W, (size_t)e * cols + c);
        out[c] = a;
    }
    __syncthreads();
}

// out[e] = sum_c x[c] W[e * cols + c] (the product with the transposed matrix): one wave per row e
template <typename T>
__device__ void wgl_dense_t(const float *x, const T *W, int rows, int cols, float *out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int e = wave; e < rows; e += kThreads / 64) {
        float a = 0.f;
        for (int c = lane; c < cols; c += 64) a += x[c] * load_f(W, (size_t)e * cols + c);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
        if (lane == 0) out[e] = a;
    }
    __syncthreads();
}

// xhat = (x - mean) / sqrt(var + eps) into xh, xhat * g + b into out (LDS, may alias x); returns 1 / sigma
template <typename T>
__device__ float wgl_layer_norm(const float *x, int m, const T *g, const T *b, float *xh, float *out, float *red)
{
    float a = 0.f;
    for (int e = threadIdx.x; e < m; e += kThreads) a += x[e];
    const float mean = wg_sum(a, red) / (float)m;
    a = 0.f;
    for (int e = threadIdx.x; e < m; e += kThreads) a += (x[e] - mean) * (x[e] - mean);
    const float inv = rsqrtf(wg_sum(a, red) / (float)m + 1e-6f);
    for (int e = threadIdx.x; e < m; e += kThreads) {
        const float xv = (x[e] - mean) * inv;
        xh[e] = xv;
        out[e] = xv * load_f(g, e) + load_f(b, e);
    }
    __syncthreads();
    return inv;
}

// dy (LDS, m entries: the gradient of the normalisation's output) -> gradient of its input, in
// place; lg / lb (staging rows, or null) receive dy * xhat and dy
template <typename T>
__device__ void wgl_layer_norm_bwd(float *dy, const float *xh, int m, const T *g, float inv, float *lg, float *lb,
                                   float *red)
{
    float a = 0.f, c = 0.f;
    for (int e = threadIdx.x; e < m; e += kThreads) {
        const float v = dy[e];
        if (lg) { lg[e] = v * xh[e]; lb[e] = v; }
        const float dx = v * load_f(g, e);
        dy[e] = dx;
        a += dx;
        c += dx * xh[e];
    }
    const float m1 = wg_sum(a, red) / (float)m, m2 = wg_sum(c, red) / (float)m;
    for (int e = threadIdx.x; e < m; e += kThreads) dy[e] = inv * (dy[e] - m1 - xh[e] * m2);
    __syncthreads();
}

template <typename T>
struct NetParams {
    const T *g1, *b1, *W1, *g2, *b2, *W2, *W3, *W4;
    __device__ NetParams(const T *P, int win, int r)
    {
        const size_t hid = 8 * (size_t)r;
        g1 = P; b1 = g1 + win; W1 = b1 + win;
        g2 = W1 + (size_t)win * hid; b2 = g2 + hid; W2 = b2 + hid;
        W3 = W2 + hid * r; W4 = W3 + (size_t)r * hid;
    }
};

// out = f(inp) for one network; with KEEP the quantities the reverse pass reads stay in L
// (a1, xh1, xh2, a3, u2; inv[0], inv[1]) and, where st is given, its layer inputs go to staging.
template <typename T, bool KEEP>
__device__ void wgl_net_fwd(const float *inp, int win, int r, const T *P, float *out, LearnedLds &L, float *inv,
                            float *st, const NetStage &ns, size_t li)
{
    const int hid = 8 * r, tid = threadIdx.x;
    const NetParams<T> np(P, win, r);
    const float i1 = wgl_layer_norm(inp, win, np.g1, np.b1, L.xh1, L.u, L.red);
    wgl_dense(L.u, win, np.W1, hid, L.a1);
    for (int c = tid; c < hid; c += kThreads) L.s1[c] = gelu_tanh_f(L.a1[c]);
    __syncthreads();
    const float i2 = wgl_layer_norm(L.s1, hid, np.g2, np.b2, L.xh2, L.s1, L.red);      // s1 = LN-2 output
    wgl_dense(L.s1, hid, np.W2, r, L.u2);
    if (KEEP && st) {
        for (int e = tid; e < win; e += kThreads) st[ns.A1 + li * win + e] = L.u[e];
        for (int c = tid; c < hid; c += kThreads) st[ns.A2 + li * hid + c] = L.s1[c];
        for (int e = tid; e < r; e += kThreads) st[ns.A3 + li * r + e] = L.u2[e];
    }
    wgl_dense(L.u2, r, np.W3, hid, L.a3);
    for (int c = tid; c < hid; c += kThreads) {
        const float hv = gelu_tanh_f(L.a3[c]);
        L.s1[c] = hv;
        if (KEEP && st) st[ns.A4 + li * hid + c] = hv;
    }
    __syncthreads();
    if (!KEEP) wgl_dense(L.s1, hid, np.W4, r, out);
    if (KEEP) { inv[0] = i1; inv[1] = i2; }
}

// Reverse pass of one network for the row whose forward quantities wgl_net_fwd<KEEP> left in L:
// df (LDS, r) = gradient of its output; dinp (LDS, win) += gradient of its input.
template <typename T>
__device__ void wgl_net_bwd(const float *df, int win, int r, const T *P, float *dinp, LearnedLds &L,
                            const float *inv, float *st, const NetStage &ns, size_t li)
{
    const int hid = 8 * r, tid = threadIdx.x;
    const NetParams<T> np(P, win, r);
    if (st)
        for (int e = tid; e < r; e += kThreads) st[ns.D4 + li * r + e] = df[e];
    wgl_dense_t(df, np.W4, hid, r, L.s1);                          // d(gelu 3 output)
    for (int c = tid; c < hid; c += kThreads) {
        const float v = L.s1[c] * gelu_tanh_grad_f(L.a3[c]);
        L.s1[c] = v;
        if (st) st[ns.D3 + li * hid + c] = v;
    }
    __syncthreads();
    wgl_dense_t(L.s1, np.W3, r, hid, L.du2);
    if (st)
        for (int e = tid; e < r; e += kThreads) st[ns.D2 + li * r + e] = L.du2[e];
    wgl_dense_t(L.du2, np.W2, hid, r, L.s1);                       // d(LN-2 output)
    wgl_layer_norm_bwd(L.s1, L.xh2, hid, np.g2, inv[1], st ? st + ns.LG2 + li * hid : nullptr,
                       st ? st + ns.LB2 + li * hid : nullptr, L.red);
    for (int c = tid; c < hid; c += kThreads) {
        const float v = L.s1[c] * gelu_tanh_grad_f(L.a1[c]);
        L.s1[c] = v;
        if (st) st[ns.D1 + li * hid + c] = v;
    }
    __syncthreads();
    wgl_dense_t(L.s1, np.W1, win, hid, L.tw);                      // d(LN-1 output)
    wgl_layer_norm_bwd(L.tw, L.xh1, win, np.g1, inv[0], st ? st + ns.LG1 + li * win : nullptr,
                       st ? st + ns.LB1 + li * win : nullptr, L.red);
    for (int e = tid; e < win; e += kThreads) dinp[e] += L.tw[e];
    __syncthreads();
}

// Rows row0 .. row0 + gridDim.x - 1 (one per workgroup, all of one parameter set P0): dX = direct
// + (d m / d x)^T dM; stage (or null): the chunk's staging, RC rows per array.
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_sketch_learned_kernel(
    const T *__restrict__ X, const T *__restrict__ P0, const float *__restrict__ dM,
    const float *__restrict__ direct, T *__restrict__ dX, long long row0, int RC, int d, int r, int p,
    float *__restrict__ stage)
{
    __shared__ LearnedLds L;
    __shared__ float xs[PSF_MAX_DIM], dxs[PSF_MAX_DIM], df[PSF_MAX_DIM];
    __shared__ float f[6][PSF_MAX_DIM], mn[2][PSF_MAX_DIM], tn[2][PSF_MAX_DIM], dmn[2][PSF_MAX_DIM];
    const int tid = threadIdx.x;
    const size_t li = blockIdx.x, row = (size_t)row0 + li;
    const float sr = sqrtf((float)r);
    if (tid < d) { xs[tid] = load_f(X, row * d + tid); dxs[tid] = direct[row * d + tid]; }
    if (tid < r) { dmn[0][tid] = 0.f; dmn[1][tid] = 0.f; }
    __syncthreads();
    float inv[2];
    // staging layout and parameter offset of network k
    auto locate = [&](int k, NetStage &ns, size_t &p_at) {
        size_t base = 0;
        p_at = 0;
        for (int j = 0;; ++j) {
            const int win = learned_net_win(j, d, r, p);
            ns = net_stage(base, (size_t)RC, win, r);
            if (j == k) return;
            base = ns.end;
            p_at += learned_net_len(win, r);
        }
    };
    auto value = [&](int k, const float *inp, int win) {
        NetStage ns;
        size_t p_at;
        locate(k, ns, p_at);
        wgl_net_fwd<T, false>(inp, win, r, P0 + p_at, f[k], L, inv, nullptr, ns, li);
    };
    // values of every network and node
    for (int k = 0; k < p / 2; ++k) value(k, xs, d);
    if (p == 8) {
        if (tid < r) {
            for (int j = 0; j < 2; ++j) {
                const float th = tanhf(f[2 * j][tid] * f[2 * j + 1][tid] / sr);
                tn[j][tid] = th;
                mn[j][tid] = sr * th;
            }
        }
        __syncthreads();
        value(4, mn[0], r);
        value(5, mn[1], r);
    }
    // the root, then down
    const int ra = p == 8 ? 4 : 0, rb = ra + 1;
    float dz = 0.f;
    if (tid < r) {
        const float th = tanhf(f[ra][tid] * f[rb][tid] / sr);
        dz = dM[row * r + tid] * (1.0f - th * th);
    }
    auto through = [&](int k, const float *inp, int win, float factor_of, float *dinp) {
        // df = dz * (value of the sibling network)
        if (tid < r) df[tid] = dz * factor_of;
        __syncthreads();
        NetStage ns;
        size_t p_at;
        locate(k, ns, p_at);
        wgl_net_fwd<T, true>(inp, win, r, P0 + p_at, nullptr, L, inv, stage, ns, li);
        wgl_net_bwd<T>(df, win, r, P0 + p_at, dinp, L, inv, stage, ns, li);
    };
    if (p == 8) {
        through(4, mn[0], r, tid < r ? f[5][tid] : 0.f, dmn[0]);
        through(5, mn[1], r, tid < r ? f[4][tid] : 0.f, dmn[1]);
        for (int j = 0; j < 2; ++j) {
            if (tid < r) dz = dmn[j][tid] * (1.0f - tn[j][tid] * tn[j][tid]);
            through(2 * j, xs, d, tid < r ? f[2 * j + 1][tid] : 0.f, dxs);
            through(2 * j + 1, xs, d, tid < r ? f[2 * j][tid] : 0.f, dxs);
        }
    } else {
        through(0, xs, d, tid < r ? f[1][tid] : 0.f, dxs);
        through(1, xs, d, tid < r ? f[0][tid] : 0.f, dxs);
    }
    if (tid < d) store_f(dX, row * d + tid, dxs[tid]);
}

// The sums over rows run in slices of kSliceRows rows (blockIdx.z): a slice leaves its part of
// every parameter in its own copy of the network's blob, bwd_param_reduce then adds the slices to
// the gradient in order.  (The outputs are small and the sums long: without slices a launch has
// a handful of workgroups.)
constexpr int kSliceRows = 256, kMaxSlices = 16;

// part[z][m][c] = sum over the rows of slice z of A[row][m] * D[row][c]  (A: [nrows][mw], D: [nrows][cw])
__global__ __launch_bounds__(kThreads) void bwd_param_gemm(const float *__restrict__ A, int mw,
                                                           const float *__restrict__ D, int cw, int nrows,
                                                           float *__restrict__ part, size_t slice_stride)
{
    __shared__ float As[32][16], Ds[32][64];
    const int tid = threadIdx.x, tc = tid & 63, tg = tid >> 6;
    const int c0 = blockIdx.x * 64, m0 = blockIdx.y * 16;
    const int row_lo = blockIdx.z * kSliceRows, row_hi = min(nrows, row_lo + kSliceRows);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int r0 = row_lo; r0 < row_hi; r0 += 32) {
        __syncthreads();
        for (int idx = tid; idx < 32 * 16; idx += kThreads) {
            const int rr = idx / 16, mm = idx % 16;
            As[rr][mm] = (r0 + rr < row_hi && m0 + mm < mw) ? A[(size_t)(r0 + rr) * mw + m0 + mm] : 0.f;
        }
        for (int idx = tid; idx < 32 * 64; idx += kThreads) {
            const int rr = idx / 64, cc = idx % 64;
            Ds[rr][cc] = (r0 + rr < row_hi && c0 + cc < cw) ? D[(size_t)(r0 + rr) * cw + c0 + cc] : 0.f;
        }
        __syncthreads();
        for (int rr = 0; rr < 32; ++rr) {
            const float dv = Ds[rr][tc];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] += As[rr][tg * 4 + j] * dv;
        }
    }
    float *out = part + (size_t)blockIdx.z * slice_stride;
    if (c0 + tc < cw)
        for (int j = 0; j < 4; ++j)
            if (m0 + tg * 4 + j < mw) out[(size_t)(m0 + tg * 4 + j) * cw + c0 + tc] = acc[j];
}

// part[z][c] = sum over the rows of slice z of X[row][c]
__global__ __launch_bounds__(kThreads) void bwd_param_colsum(const float *__restrict__ X, int w, int nrows,
                                                             float *__restrict__ part, size_t slice_stride)
{
    const int c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= w) return;
    const int row_lo = blockIdx.z * kSliceRows, row_hi = min(nrows, row_lo + kSliceRows);
    float a = 0.f;
    for (int rr = row_lo; rr < row_hi; ++rr) a += X[(size_t)rr * w + c];
    part[(size_t)blockIdx.z * slice_stride + c] = a;
}

// g[i] += part[0][i] + part[1][i] + ... in that order
__global__ __launch_bounds__(kThreads) void bwd_param_reduce(const float *__restrict__ part, size_t count,
                                                             int slices, size_t slice_stride, float *__restrict__ g)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= count) return;
    float a = g[i];
    for (int z = 0; z < slices; ++z) a += part[(size_t)z * slice_stride + i];
    g[i] = a;
}

__global__ __launch_bounds__(kThreads) void bwd_fill_kernel(float *__restrict__ p, size_t count)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// staging floats per row over all networks of one set
size_t learned_stage_floats_per_row(const Problem &pb)
{
    size_t at = 0;
    for (int k = 0; k < pb.p - 2; ++k) at = net_stage(at, 1, learned_net_win(k, pb.d, pb.r, pb.p), pb.r).end;
    return at;
}

// rows per chunk: at most 128 MB of staging, at most 4096 rows, at least 64
int learned_chunk_rows(const Problem &pb)
{
    const size_t per_row = learned_stage_floats_per_row(pb) * 4;
    size_t rc = ((size_t)128 << 20) / (per_row ? per_row : 1);
    if (rc > 4096) rc = 4096;
    if (rc < 64) rc = 64;
    const size_t seg = pb.per_head ? (size_t)pb.n : (size_t)pb.units * pb.n;
    return (int)(rc < seg ? rc : seg);
}

// dX = direct + J^T dM through Algorithm 2 for every row of X; dG (or null) += the parameter gradient
template <typename T>
psf_status learned_sketch_bwd(const Problem &pb, const void *X, const void *G, const float *dM,
                              const float *direct, void *dX, float *dG, float *stage, float *part, hipStream_t s)
{
    const int RC = learned_chunk_rows(pb), nets = pb.p - 2, r = pb.r, hid = 8 * pb.r;
    const size_t slice_stride = learned_net_len(pb.d > r ? pb.d : r, r);      // the longest network blob
    const size_t rows = (size_t)pb.units * pb.n;
    const size_t seg_rows = pb.per_head ? (size_t)pb.n : rows;
    for (size_t seg0 = 0; seg0 < rows; seg0 += seg_rows) {
        const size_t set = pb.per_head ? (seg0 / pb.n) % pb.heads : 0;
        const T *P0 = (const T *)G + set * pb.g_len;
        for (size_t c0 = 0; c0 < seg_rows; c0 += RC) {
            const int nrows = (int)(seg_rows - c0 < (size_t)RC ? seg_rows - c0 : (size_t)RC);
            hipLaunchKernelGGL(bwd_sketch_learned_kernel<T>, dim3(nrows), dim3(kThreads), 0, s, (const T *)X, P0, dM,
                               direct, (T *)dX, (long long)(seg0 + c0), RC, pb.d, r, pb.p, dG ? stage : nullptr);
            PSF_LAUNCH_CHECK();
            if (!dG) continue;
            size_t base = 0, p_at = 0;
            for (int k = 0; k < nets; ++k) {
                const int win = learned_net_win(k, pb.d, r, pb.p);
                const NetStage ns = net_stage(base, (size_t)RC, win, r);
                base = ns.end;
                float *g = part;                               // slice 0 of this network's blob
                float *g1 = g, *b1 = g1 + win, *W1 = b1 + win;
                float *g2 = W1 + (size_t)win * hid, *b2 = g2 + hid, *W2 = b2 + hid;
                float *W3 = W2 + (size_t)hid * r, *W4 = W3 + (size_t)r * hid;
                const size_t net_len = learned_net_len(win, r);
                const int slices = (nrows + kSliceRows - 1) / kSliceRows;      // <= kMaxSlices: RC <= 4096
                auto gemm = [&](size_t a_off, int mw, size_t d_off, int cw, float *dW) {
                    hipLaunchKernelGGL(bwd_param_gemm, dim3((cw + 63) / 64, (mw + 15) / 16, slices), dim3(kThreads), 0,
                                       s, stage + a_off, mw, stage + d_off, cw, nrows, dW, slice_stride);
                };
                auto colsum = [&](size_t x_off, int w, float *out) {
                    hipLaunchKernelGGL(bwd_param_colsum, dim3((w + kThreads - 1) / kThreads, 1, slices), dim3(kThreads),
                                       0, s, stage + x_off, w, nrows, out, slice_stride);
                };
                colsum(ns.LG1, win, g1);
                colsum(ns.LB1, win, b1);
                gemm(ns.A1, win, ns.D1, hid, W1);
                colsum(ns.LG2, hid, g2);
                colsum(ns.LB2, hid, b2);
                gemm(ns.A2, hid, ns.D2, r, W2);
                gemm(ns.A3, r, ns.D3, hid, W3);
                gemm(ns.A4, hid, ns.D4, r, W4);
                hipLaunchKernelGGL(bwd_param_reduce, dim3((unsigned)((net_len + kThreads - 1) / kThreads)),
                                   dim3(kThreads), 0, s, part, net_len, slices, slice_stride,
                                   dG + set * pb.g_len + p_at);
                p_at += net_len;
                PSF_LAUNCH_CHECK();
            }
        }
    }
    return PSF_OK;
}

struct BwdWs {
    float *MQ, *MK, *CV, *GC, *Z, *RB, *dMQ, *dMK, *dQd, *dKd;
    float *LS, *LP;                              // learned sketches: staging of one chunk of rows; slices of one network's sums
    size_t total;
};

BwdWs carve_bwd(const Problem &pb, void *ws)
{
    BwdWs w;
    const size_t rows = (size_t)pb.units * pb.n, kc = (size_t)pb.dv + 1;
    size_t off = 0;
    char *base = (char *)ws;
    auto take = [&](size_t floats) { char *p = base + off; off += align_up(floats * 4, 256); return (float *)p; };
    w.MQ = take(rows * pb.mcols);
    w.MK = take(rows * pb.mcols);
    w.CV = take(rows * kc);
    w.GC = take(rows * kc);
    w.Z = take((size_t)pb.units * pb.t * (size_t)pb.F * kc);
    w.RB = take((size_t)pb.units * pb.t * (size_t)pb.F * kc);
    w.dMQ = take(rows * pb.mcols);
    w.dMK = take(rows * pb.mcols);
    w.dQd = take(rows * pb.d);
    w.dKd = take(rows * pb.d);
    w.LS = take(pb.learned ? (size_t)learned_chunk_rows(pb) * learned_stage_floats_per_row(pb) : 0);
    w.LP = take(pb.learned ? (size_t)kMaxSlices * learned_net_len(pb.d > pb.r ? pb.d : pb.r, pb.r) : 0);
    w.total = off;
    return w;
}

template <typename T>
psf_status bwd_launch(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                      const void *dO, void *dQ, void *dK, void *dV, float *dG, void *ws, hipStream_t s,
                      StageTimer *tm)
{
    BwdWs w = carve_bwd(pb, ws);
    const size_t rows = (size_t)pb.units * pb.n;
    const int kc = pb.dv + 1;
    const int le = pb.local_exact ? 1 : 0;
    psf_status st = general_sketch_f32(pb, Q, G, w.MQ, s);
    if (st != PSF_OK) return st;
    st = general_sketch_f32(pb, K, G, w.MK, s);
    if (st != PSF_OK) return st;
    hipLaunchKernelGGL(bwd_cv_kernel<T>, dim3((unsigned)((rows * kc + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, s, (const T *)V, w.CV, rows, pb.dv);
    PSF_LAUNCH_CHECK();
    if (tm) tm->mark();                                   // stage: sketches

    const dim3 sgrid((unsigned)((pb.F + kStateFeat - 1) / kStateFeat), (unsigned)pb.t, (unsigned)pb.units);
    const size_t per_block = (size_t)pb.F * kc;
    const unsigned scan_grid = (unsigned)(((size_t)pb.units * per_block + kThreads - 1) / kThreads);
    if (pb.t > 1) {
        hipLaunchKernelGGL(bwd_state_kernel, sgrid, dim3(kThreads), 0, s, w.MK, w.CV, w.Z, pb.n, kc, pb.b,
                           pb.t, pb.mcols, pb.F);
        PSF_LAUNCH_CHECK();
        hipLaunchKernelGGL(bwd_scan_kernel, dim3(scan_grid), dim3(kThreads), 0, s, w.Z, pb.units, pb.t,
                           per_block, 0);
        PSF_LAUNCH_CHECK();
    }
    int RT = kRows;                                       // tokens per workgroup, all in one block
    while (pb.b % RT != 0) RT /= 2;
    const dim3 rgrid((unsigned)(pb.n / RT), (unsigned)pb.units);
    const int wa = pb.local_exact ? pb.d : pb.mcols;
    const size_t lds_rows = rows_lds(nullptr, pb.d, kc, pb.mcols, wa, nullptr, nullptr, nullptr, nullptr, nullptr);
    const size_t lds_q = q_lds(nullptr, pb.d, kc, pb.mcols, wa, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    const size_t lds_k = k_lds(nullptr, pb.d, kc, pb.mcols, wa, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                               nullptr);
    // the largest admitted sizes (d = dv = r = 256) need more than the default dynamic LDS limit
    PSF_HIP_TRY(hipFuncSetAttribute((const void *)bwd_rows_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds_rows));
    PSF_HIP_TRY(hipFuncSetAttribute((const void *)bwd_q_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds_q));
    PSF_HIP_TRY(hipFuncSetAttribute((const void *)bwd_k_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds_k));
    hipLaunchKernelGGL(bwd_rows_kernel<T>, rgrid, dim3(kThreads), lds_rows, s, w.MQ, w.MK, (const T *)Q,
                       (const T *)K, w.CV, w.Z, (const T *)dO, w.GC, pb.n, pb.d, pb.dv, pb.p, pb.b, pb.t,
                       pb.mcols, pb.F, le, RT);
    PSF_LAUNCH_CHECK();
    if (tm) tm->mark();                                   // stage: forward rows

    if (pb.t > 1) {
        hipLaunchKernelGGL(bwd_state_kernel, sgrid, dim3(kThreads), 0, s, w.MQ, w.GC, w.RB, pb.n, kc, pb.b,
                           pb.t, pb.mcols, pb.F);
        PSF_LAUNCH_CHECK();
        hipLaunchKernelGGL(bwd_scan_kernel, dim3(scan_grid), dim3(kThreads), 0, s, w.RB, pb.units, pb.t,
                           per_block, 1);
        PSF_LAUNCH_CHECK();
    }
    if (tm) tm->mark();                                   // stage: reverse states

    hipLaunchKernelGGL(bwd_q_kernel<T>, rgrid, dim3(kThreads), lds_q, s, w.MQ, w.MK, (const T *)Q, (const T *)K,
                       w.CV, w.GC, w.Z, w.dMQ, w.dQd, pb.n, pb.d, pb.dv, pb.p, pb.b, pb.t, pb.mcols, pb.F, le, RT);
    PSF_LAUNCH_CHECK();
    if (tm) tm->mark();                                   // stage: query side
    hipLaunchKernelGGL(bwd_k_kernel<T>, rgrid, dim3(kThreads), lds_k, s, w.MQ, w.MK, (const T *)Q, (const T *)K,
                       w.CV, w.GC, w.RB, w.dMK, w.dKd, (T *)dV, pb.n, pb.d, pb.dv, pb.p, pb.b, pb.t,
                       pb.mcols, pb.F, le, RT);
    PSF_LAUNCH_CHECK();
    if (tm) tm->mark();                                   // stage: key side

    if (pb.learned) {
        if (dG) {
            const size_t count = (size_t)(pb.per_head ? pb.heads : 1) * pb.g_len;
            hipLaunchKernelGGL(bwd_fill_kernel, dim3((unsigned)((count + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                               s, dG, count);
            PSF_LAUNCH_CHECK();
        }
        st = learned_sketch_bwd<T>(pb, Q, G, w.dMQ, w.dQd, dQ, dG, w.LS, w.LP, s);
        if (st != PSF_OK) return st;
        st = learned_sketch_bwd<T>(pb, K, G, w.dMK, w.dKd, dK, dG, w.LS, w.LP, s);
        if (st != PSF_OK) return st;
        if (tm) tm->mark();                               // stage: sketch gradient
        return PSF_OK;
    }
    const int grid = (int)(rows < 65536 ? rows : 65536);
    hipLaunchKernelGGL(bwd_sketch_kernel<T>, dim3(grid), dim3(kThreads), 0, s, (const T *)Q, (const T *)G,
                       w.dMQ, w.dQd, (T *)dQ, (long long)rows, pb.n, pb.heads, pb.per_head ? 1 : 0, pb.d,
                       pb.r, pb.p, pb.g_len);
    PSF_LAUNCH_CHECK();
    hipLaunchKernelGGL(bwd_sketch_kernel<T>, dim3(grid), dim3(kThreads), 0, s, (const T *)K, (const T *)G,
                       w.dMK, w.dKd, (T *)dK, (long long)rows, pb.n, pb.heads, pb.per_head ? 1 : 0, pb.d,
                       pb.r, pb.p, pb.g_len);
    PSF_LAUNCH_CHECK();
    if (tm) tm->mark();                                   // stage: sketch gradient
    return PSF_OK;
}

}  // namespace

// Algorithm 1's reverse alone: dX = direct + J_m(X)^T dM for rows of X (storage type of pb), with
// dM [rows][mcols] and direct [rows][d] fp32.
psf_status general_sketch_bwd(const Problem &pb, const void *X, const void *G, const float *dM,
                              const float *direct, void *dX, hipStream_t s)
{
    const size_t rows = (size_t)pb.units * pb.n;
    const int grid = (int)(rows < 65536 ? rows : 65536);
    if (pb.bf16)
        hipLaunchKernelGGL(bwd_sketch_kernel<bf16_t>, dim3(grid), dim3(kThreads), 0, s, (const bf16_t *)X,
                           (const bf16_t *)G, dM, direct, (bf16_t *)dX, (long long)rows, pb.n, pb.heads,
                           pb.per_head ? 1 : 0, pb.d, pb.r, pb.p, pb.g_len);
    else
        hipLaunchKernelGGL(bwd_sketch_kernel<float>, dim3(grid), dim3(kThreads), 0, s, (const float *)X,
                           (const float *)G, dM, direct, (float *)dX, (long long)rows, pb.n, pb.heads,
                           pb.per_head ? 1 : 0, pb.d, pb.r, pb.p, pb.g_len);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}

bool general_bwd_supported(const Problem &pb)
{
    // explicit x^{(x)p} features have no backward here; the feature staging assumes F and a
    // block fit the chunked LDS loops (any size) and the 32-bit feature index of one pass
    return !pb.exact_feat && pb.F <= PSF_MAX_FEATURES;
}

size_t general_bwd_workspace_bytes(const Problem &pb) { return carve_bwd(pb, nullptr).total; }

psf_status general_attn_bwd(const Problem &pb, const void *Q, const void *K, const void *V,
                            const void *G, const void *dO, void *dQ, void *dK, void *dV, void *ws,
                            hipStream_t s, StageTimer *tm, float *dG)
{
    return pb.bf16 ? bwd_launch<bf16_t>(pb, Q, K, V, G, dO, dQ, dK, dV, dG, ws, s, tm)
                   : bwd_launch<float>(pb, Q, K, V, G, dO, dQ, dK, dV, dG, ws, s, tm);
}

}  // namespace psf
