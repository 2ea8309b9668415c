// Token-by-token evaluation of causal Polysketch attention (PolySketchFormer, arXiv 2310.01655):
// the recurrent form the paper points to when it notes that the state kept for generation does
// not grow with the context (Section 5).  One step consumes the (q, k, v) of position `pos` and
// returns row `pos` of the attention of Section 3, identical to what the block algorithm of
// Sections 3.1 / 3.2 with block size b returns for the sequence so far:
//   o = (phi'(q)^T Z + sum_{j in current block, j <= pos} w_j [v_j | 1]) -> N / (1 + S)
// where Z = sum over the *completed* blocks of phi'(k_j) [v_j | 1]^T is the prefix state Z_l of
// Section 3.1 and w_j = <q, k_j>^p (Section 3.2) or <m(q), m(k_j)>^2 (Section 3.1) inside the
// current block.  When a block completes, its keys are folded into Z.
//
// State per (batch, head) unit, all fp32, caller-owned:
//   ZV [F][dv] and ZD [F]: the value columns and the "ones" column of Z (F = mcols^2 features),
//   kept apart so that rows of ZV are aligned and a step streams them with full-width loads;
//   then the current block's cache: CK [b][d] keys and CV [b][dv] values in the storage type
//   of the call (fp32 or bf16), CM [b][mcols] sketches m(k) in fp32.  After the units come the scratch areas: m(q), m(k) of the new token [units][mcols]
//   each and the partial sums of the state product [units][kSlices][dv + 1].
// A step is bound by reading Z once (F * (dv + 1) * 4 bytes per unit) from HBM.
#include "psf_internal.h"

namespace psf {
namespace {

constexpr int kThreads = 256;
constexpr int kSlices = 16;        // workgroups per unit in the state product

struct DecodeLayout {
    size_t zv, zd, ck, cv, cm, per_unit;     // float offsets inside one unit, floats per unit
    size_t mq, mk, part, total;              // float offsets of the scratch areas, total floats
};

DecodeLayout decode_layout(const Problem &pb)
{
    DecodeLayout L;
    auto up = [](size_t v) { return (v + 63) / 64 * 64; };            // 256-byte pieces
    L.zv = 0;
    L.zd = up((size_t)pb.F * pb.dv);
    const size_t per_float = pb.bf16 ? 2 : 1;                         // cached keys / values keep the storage type
    L.ck = L.zd + up((size_t)pb.F);
    L.cv = L.ck + up(((size_t)pb.b * pb.d + per_float - 1) / per_float);
    L.cm = L.cv + up(((size_t)pb.b * pb.dv + per_float - 1) / per_float);
    L.per_unit = L.cm + up((size_t)pb.b * pb.mcols);
    L.mq = L.per_unit * pb.units;
    L.mk = L.mq + up((size_t)pb.units * pb.mcols);
    L.part = L.mk + up((size_t)pb.units * pb.mcols);
    L.total = L.part + up((size_t)pb.units * kSlices * (pb.dv + 1));
    return L;
}

__device__ __forceinline__ int pow2_at_least(int v, int lo, int hi)
{
    int p = lo;
    while (p < v && p < hi) p *= 2;
    return p;
}

__device__ __forceinline__ float4 load4_f(const float *p) { return *(const float4 *)p; }
__device__ __forceinline__ float4 load4_f(const bf16_t *p)
{
    const uint2 w = *(const uint2 *)p;
    return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                       __uint_as_float(w.y & 0xffff0000u));
}

__global__ __launch_bounds__(kThreads) void dec_zero_kernel(float *__restrict__ p, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += (size_t)gridDim.x * kThreads)
        p[i] = 0.f;
}

// part[u][s][c] = the share of slice s in row [N | S] of the new token:
//   cross-block: sum over the features f of the slice of phi'(q)[f] ZV[f][c] (c < dv) and, at
//   c = dv, of phi'(q)[f] ZD[f] (only once a block is complete: have_state); phi'(q) of the slice
//   sits in LDS; thread (c, g) walks the rows g, g + groups, ... four at a time, so a wave reads
//   whole contiguous rows of ZV;
//   in-block: the slice's share of the `slot` tokens cached since the last block boundary,
//   sum_j w_j [v_j | 1] with the weights of Section 3.2 (or 3.1).  The new token itself is not in
//   the cache yet: its own pair is added by dec_finish_kernel.
template <typename T>
__global__ __launch_bounds__(kThreads) void dec_state_kernel(const T *__restrict__ q,
                                                             const float *__restrict__ state,
                                                             const float *__restrict__ mq_new,
                                                             float *__restrict__ part, DecodeLayout L, int d,
                                                             int dv, int p, int mcols, long long F, int slot,
                                                             int have_state, int local_exact)
{
    constexpr int kMaxPer = 4096;                          // F / kSlices <= 65536 / 16
    __shared__ float mq[PSF_MAX_DIM], qs[PSF_MAX_DIM], phi[kMaxPer], red[kThreads], w[kThreads], rowp[PSF_MAX_DIM + 1];
    const int u = blockIdx.y, sl = blockIdx.x, tid = threadIdx.x, kc = dv + 1;
    const float *su = state + (size_t)u * L.per_unit;
    for (int e = tid; e < mcols; e += kThreads) mq[e] = mq_new[(size_t)u * mcols + e];
    const int wa = local_exact ? d : mcols;
    for (int e = tid; e < wa; e += kThreads)
        qs[e] = local_exact ? load_f(q, (size_t)u * d + e) : mq_new[(size_t)u * mcols + e];
    for (int c = tid; c < kc; c += kThreads) rowp[c] = 0.f;
    __syncthreads();
    const int dvp = pow2_at_least(dv, 32, kThreads), groups = kThreads / dvp;
    float *out = part + ((size_t)u * kSlices + sl) * kc;

    if (have_state) {
        const long long per = (F + kSlices - 1) / kSlices;
        const long long f_beg = sl * per;
        const int nf = (int)max(0LL, min(F, f_beg + per) - f_beg);
        for (int ff = tid; ff < nf; ff += kThreads) {
            const long long f = f_beg + ff;
            phi[ff] = mq[f / mcols] * mq[f % mcols];
        }
        __syncthreads();
        const float *zv = su + L.zv + (size_t)f_beg * dv;
        const float *zd = su + L.zd + f_beg;
        if ((dv & 3) == 0 && dv <= 4 * kThreads) {
            // four columns per thread (16-byte loads), consecutive lane groups on consecutive rows:
            // a wave reads contiguous kilobytes; eight rows in flight per thread
            const int c4n = dv / 4, c4p = pow2_at_least(c4n, 1, kThreads), grp4 = kThreads / c4p;
            const int c4 = tid % c4p, g = tid / c4p;
            float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0;
            if (c4 < c4n) {
                const float4 *z4 = (const float4 *)zv + c4;
                int ff = g;
                for (; ff + 7 * grp4 < nf; ff += 8 * grp4) {
                    float4 zr[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) zr[i] = z4[(size_t)(ff + i * grp4) * c4n];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float ph = phi[ff + i * grp4];
                        float4 &acc4 = (i & 1) ? s1 : s0;
                        acc4.x += ph * zr[i].x; acc4.y += ph * zr[i].y; acc4.z += ph * zr[i].z; acc4.w += ph * zr[i].w;
                    }
                }
                for (; ff < nf; ff += grp4) {
                    const float4 zr = z4[(size_t)ff * c4n];
                    const float ph = phi[ff];
                    s0.x += ph * zr.x; s0.y += ph * zr.y; s0.z += ph * zr.z; s0.w += ph * zr.w;
                }
            }
            float *red4 = phi;                              // phi of the slice is no longer needed after this
            // (the ones column below reads phi: do it first)
            float a1c = 0.f;
            for (int ff = tid; ff < nf; ff += kThreads) a1c += phi[ff] * zd[ff];
            __syncthreads();
            red[tid] = a1c;
            red4[4 * tid + 0] = s0.x + s1.x; red4[4 * tid + 1] = s0.y + s1.y;
            red4[4 * tid + 2] = s0.z + s1.z; red4[4 * tid + 3] = s0.w + s1.w;
            __syncthreads();
            if (tid < dv) {
                const int cc4 = tid / 4, j4 = tid % 4;
                float sacc = 0.f;
                for (int q2 = 0; q2 < grp4; ++q2) sacc += red4[4 * (q2 * c4p + cc4) + j4];
                rowp[tid] = sacc;
            }
            if (tid == 0) {
                float sacc = 0.f;
                for (int q2 = 0; q2 < kThreads; ++q2) sacc += red[q2];
                rowp[dv] = sacc;
            }
        } else {
            for (int c0 = 0; c0 < dv; c0 += dvp) {
                const int c = c0 + tid % dvp, g = tid / dvp;
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
                if (c < dv) {
                    int ff = g;
                    for (; ff + 7 * groups < nf; ff += 8 * groups) {          // eight rows in flight per thread
                        const float z0 = zv[(size_t)ff * dv + c], z1 = zv[(size_t)(ff + groups) * dv + c];
                        const float z2 = zv[(size_t)(ff + 2 * groups) * dv + c], z3 = zv[(size_t)(ff + 3 * groups) * dv + c];
                        const float z4 = zv[(size_t)(ff + 4 * groups) * dv + c], z5 = zv[(size_t)(ff + 5 * groups) * dv + c];
                        const float z6 = zv[(size_t)(ff + 6 * groups) * dv + c], z7 = zv[(size_t)(ff + 7 * groups) * dv + c];
                        a0 += phi[ff] * z0 + phi[ff + 4 * groups] * z4;
                        a1 += phi[ff + groups] * z1 + phi[ff + 5 * groups] * z5;
                        a2 += phi[ff + 2 * groups] * z2 + phi[ff + 6 * groups] * z6;
                        a3 += phi[ff + 3 * groups] * z3 + phi[ff + 7 * groups] * z7;
                    }
                    for (; ff < nf; ff += groups) a0 += phi[ff] * zv[(size_t)ff * dv + c];
                }
                __syncthreads();
                red[tid] = (a0 + a1) + (a2 + a3);
                __syncthreads();
                if (tid < dvp && c0 + tid < dv) {
                    float sacc = 0.f;
                    for (int q2 = 0; q2 < groups; ++q2) sacc += red[q2 * dvp + tid];
                    rowp[c0 + tid] = sacc;
                }
            }
            // the "ones" column
            float a = 0.f;
            for (int ff = tid; ff < nf; ff += kThreads) a += phi[ff] * zd[ff];
            __syncthreads();
            red[tid] = a;
            __syncthreads();
            if (tid == 0) {
                float sacc = 0.f;
                for (int q2 = 0; q2 < kThreads; ++q2) sacc += red[q2];
                rowp[dv] = sacc;
            }
        }
    }

    // in-block: cached tokens j_beg .. j_end - 1 of this slice
    const int per_j = (slot + kSlices - 1) / kSlices;
    const int j_beg = min(slot, sl * per_j), j_end = min(slot, j_beg + per_j);
    const T *ckeys = (const T *)(su + L.ck);             // local_exact: the cached keys, storage type
    const float *mkeys = su + L.cm;                        // otherwise: their sketches
    const T *cvals = (const T *)(su + L.cv);
    for (int j0 = j_beg; j0 < j_end; j0 += kThreads) {
        const int nj = min(kThreads, j_end - j0);
        __syncthreads();
        // weights of the pass: four threads per key (consecutive lanes read consecutive pieces of
        // a cached row), 64 keys at a time
        for (int kk = 0; kk < nj; kk += kThreads / 4) {
            const int kj = kk + (tid >> 2), part4 = tid & 3;
            float sdot = 0.f;
            if (kj < nj) {
                const size_t roff = (size_t)(j0 + kj) * wa;
                if ((wa & 15) == 0) {
                    for (int e = 4 * part4; e < wa; e += 16) {
                        const float4 kv = local_exact ? load4_f(ckeys + roff + e) : load4_f(mkeys + roff + e);
                        sdot += qs[e] * kv.x + qs[e + 1] * kv.y + qs[e + 2] * kv.z + qs[e + 3] * kv.w;
                    }
                } else {
                    for (int e = part4; e < wa; e += 4)
                        sdot += qs[e] * (local_exact ? load_f(ckeys, roff + e) : mkeys[roff + e]);
                }
            }
            sdot += __shfl_xor(sdot, 1);
            sdot += __shfl_xor(sdot, 2);
            if (part4 == 0 && kj < nj) {
                float wv = sdot * sdot;
                if (local_exact) {
                    wv = 1.f;
                    for (int e = 0; e < p; ++e) wv *= sdot;
                }
                w[kj] = wv;
            }
        }
        __syncthreads();
        for (int c0 = 0; c0 < dv; c0 += dvp) {            // values: thread (c, g) takes slots g, g + groups, ...
            const int c = c0 + tid % dvp, g = tid / dvp;
            float a = 0.f;
            if (c < dv)
                for (int jj = g; jj < nj; jj += groups) a += w[jj] * load_f(cvals, (size_t)(j0 + jj) * dv + c);
            __syncthreads();
            red[tid] = a;
            __syncthreads();
            if (tid < dvp && c0 + tid < dv) {
                float sacc = 0.f;
                for (int q2 = 0; q2 < groups; ++q2) sacc += red[q2 * dvp + tid];
                rowp[c0 + tid] += sacc;
            }
        }
        if (tid == 0) {                                   // the "ones" column: sum of the weights
            float sacc = 0.f;
            for (int jj = 0; jj < nj; ++jj) sacc += w[jj];
            rowp[dv] += sacc;
        }
    }
    __syncthreads();
    for (int c = tid; c < kc; c += kThreads) out[c] = rowp[c];
}

// The new token's key, value and m(k) go into cache slot `slot`; row = sum of the slices + the
// new token's own pair; then N / (1 + S).
template <typename T>
__global__ __launch_bounds__(kThreads) void dec_finish_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                              const T *__restrict__ v,
                                                              float *__restrict__ state,
                                                              const float *__restrict__ mq_new,
                                                              const float *__restrict__ mk_new,
                                                              const float *__restrict__ part,
                                                              T *__restrict__ o, DecodeLayout L, int d,
                                                              int dv, int p, int mcols, int slot,
                                                              int local_exact)
{
    __shared__ float red[kThreads];
    __shared__ float w_self;
    const int u = blockIdx.x, tid = threadIdx.x, kc = dv + 1;
    float *su = state + (size_t)u * L.per_unit;
    T *ckeys = (T *)(su + L.ck), *cvals = (T *)(su + L.cv);
    for (int e = tid; e < d; e += kThreads) ckeys[(size_t)slot * d + e] = k[(size_t)u * d + e];
    for (int c = tid; c < dv; c += kThreads) cvals[(size_t)slot * dv + c] = v[(size_t)u * dv + c];
    for (int e = tid; e < mcols; e += kThreads) su[L.cm + (size_t)slot * mcols + e] = mk_new[(size_t)u * mcols + e];
    // own pair: <q, k>^p, or <m(q), m(k)>^2 with the sketched in-block rule
    const int wa = local_exact ? d : mcols;
    float a = 0.f;
    for (int e = tid; e < wa; e += kThreads)
        a += local_exact ? load_f(q, (size_t)u * d + e) * load_f(k, (size_t)u * d + e)
                         : mq_new[(size_t)u * mcols + e] * mk_new[(size_t)u * mcols + e];
    red[tid] = a;
    __syncthreads();
    if (tid == 0) {
        float sdot = 0.f;
        for (int q2 = 0; q2 < kThreads; ++q2) sdot += red[q2];
        float wv = sdot * sdot;
        if (local_exact) {
            wv = 1.f;
            for (int e = 0; e < p; ++e) wv *= sdot;
        }
        w_self = wv;
    }
    __syncthreads();
    float den = 1.f + w_self;
    for (int sidx = 0; sidx < kSlices; ++sidx) den += part[((size_t)u * kSlices + sidx) * kc + dv];
    for (int c = tid; c < dv; c += kThreads) {
        float acc = w_self * load_f(v, (size_t)u * dv + c);
        for (int sidx = 0; sidx < kSlices; ++sidx) acc += part[((size_t)u * kSlices + sidx) * kc + c];
        store_f(o, (size_t)u * dv + c, acc / den);
    }
}

// ZV[f][c] += sum over the b cached tokens of phi'(k_j)[f] v_j[c], ZD[f] += sum_j phi'(k_j)[f].
// Workgroup = kFoldFeat features; thread (c, g) owns the PER = kFoldFeat / groups features
// g * PER .. of column c (groups = 256 / columns per pass).
constexpr int kFoldFeat = 64, kFoldTok = 32;
template <typename T, int PER>
__global__ __launch_bounds__(kThreads) void dec_fold_kernel(float *__restrict__ state, DecodeLayout L,
                                                            int dv, int b, int mcols, long long F)
{
    __shared__ float phi[kFoldTok][kFoldFeat + 1], vt[kFoldTok][PSF_MAX_DIM];
    constexpr int groups = kFoldFeat / PER, dvp = kThreads / groups;
    const int tid = threadIdx.x, u = blockIdx.y;
    const long long f0 = (long long)blockIdx.x * kFoldFeat;
    float *su = state + (size_t)u * L.per_unit;
    for (int c0 = 0; c0 < dv; c0 += dvp) {
        const int c = c0 + tid % dvp, g = tid / dvp;
        float acc[PER];
#pragma unroll
        for (int ff = 0; ff < PER; ++ff) acc[ff] = 0.f;
        float dacc = 0.f;                                 // ZD: thread tid < kFoldFeat owns feature tid
        for (int j0 = 0; j0 < b; j0 += kFoldTok) {
            const int lim = min(kFoldTok, b - j0);
            __syncthreads();
            for (int idx = tid; idx < kFoldTok * kFoldFeat; idx += kThreads) {
                const int jj = idx / kFoldFeat, ff = idx % kFoldFeat;
                float v = 0.f;
                if (jj < lim && f0 + ff < F) {
                    const float *m = su + L.cm + (size_t)(j0 + jj) * mcols;
                    const long long f = f0 + ff;
                    v = m[f / mcols] * m[f % mcols];
                }
                phi[jj][ff] = v;
            }
            for (int idx = tid; idx < kFoldTok * dv; idx += kThreads) {
                const int jj = idx / dv, cc = idx % dv;
                vt[jj][cc] = jj < lim ? load_f((const T *)(su + L.cv), (size_t)(j0 + jj) * dv + cc) : 0.f;
            }
            __syncthreads();
            if (c < dv)
                for (int jj = 0; jj < kFoldTok; ++jj) {
                    const float vv = vt[jj][c];
#pragma unroll
                    for (int ff = 0; ff < PER; ++ff) acc[ff] += phi[jj][g * PER + ff] * vv;
                }
            if (c0 == 0 && tid < kFoldFeat)
                for (int jj = 0; jj < kFoldTok; ++jj) dacc += phi[jj][tid];
        }
        if (c < dv) {
#pragma unroll
            for (int ff = 0; ff < PER; ++ff)
                if (f0 + g * PER + ff < F) su[L.zv + (size_t)(f0 + g * PER + ff) * dv + c] += acc[ff];
        }
        if (c0 == 0 && tid < kFoldFeat && f0 + tid < F) su[L.zd + f0 + tid] += dacc;
    }
}

// The same fold on MFMA for bf16 storage (phi'(k) and v as bf16 operands, fp32 accumulation, as
// the forward state kernel does): Z[a][b'][c] += sum_j (m_j[a] m_j[b']) v_j[c].  Workgroup =
// (NA consecutive sketch rows a, unit); wave w owns the 32 x 32 tiles w, w + 4, ... (SLOTS of
// them) of each row's [mcols][dv] block.  64 tokens at a time are staged transposed
// ([column][token]) so that a lane's eight tokens of one column are neighbours; the fragments of
// m_j[b'] and of v are shared by the NA rows.
typedef __bf16 dec_bf16x8 __attribute__((ext_vector_type(8)));
typedef float dec_f32x16 __attribute__((ext_vector_type(16)));
constexpr int kFoldMfmaTok = 64, kFoldMfmaMaxM = 64, kFoldMfmaMaxDv = 128;

template <int SLOTS>
__global__ __launch_bounds__(kThreads) void dec_fold_mfma_kernel(float *__restrict__ state, DecodeLayout L,
                                                                 int dv, int b, int mcols)
{
    constexpr int TOK = kFoldMfmaTok, PITCH = TOK + 1;      // odd pitch: conflict-free column reads
    constexpr int NA = 8 / SLOTS;
    __shared__ float mts[kFoldMfmaMaxM][PITCH], vts[kFoldMfmaMaxDv][PITCH];
    const int a0 = blockIdx.x * NA, u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int x = lane & 31, h = lane >> 5;
    float *su = state + (size_t)u * L.per_unit;
    const int tiles_c = dv / 32, ntiles = (mcols / 32) * tiles_c;
    dec_f32x16 acc[SLOTS][NA];
    float drow[SLOTS][NA];
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl)
#pragma unroll
        for (int ai = 0; ai < NA; ++ai) {
            drow[sl][ai] = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[sl][ai][v] = 0.f;
        }
    for (int j0 = 0; j0 < b; j0 += TOK) {
        __syncthreads();
        for (int idx = tid; idx < TOK * mcols; idx += kThreads) {
            const int jj = idx / mcols, col = idx % mcols;
            mts[col][jj] = j0 + jj < b ? su[L.cm + (size_t)(j0 + jj) * mcols + col] : 0.f;
        }
        for (int idx = tid; idx < TOK * dv; idx += kThreads) {
            const int jj = idx / dv, c = idx % dv;
            vts[c][jj] = j0 + jj < b ? bf16_to_f32(((const bf16_t *)(su + L.cv))[(size_t)(j0 + jj) * dv + c]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int sl = 0; sl < SLOTS; ++sl) {
            const int ti = wave + 4 * sl;
            if (ti >= ntiles) break;
            const int bt = ti / tiles_c, ct = ti % tiles_c;
#pragma unroll
            for (int sstep = 0; sstep < TOK / 16; ++sstep) {
                float mb[8];
                dec_bf16x8 fb;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int tok = 16 * sstep + 8 * h + e;
                    mb[e] = mts[32 * bt + x][tok];
                    fb[e] = (__bf16)vts[32 * ct + x][tok];
                }
#pragma unroll
                for (int ai = 0; ai < NA; ++ai) {
                    dec_bf16x8 fa;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float pr = mts[a0 + ai][16 * sstep + 8 * h + e] * mb[e];
                        fa[e] = (__bf16)pr;
                        if (ct == 0) drow[sl][ai] += pr;
                    }
                    acc[sl][ai] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[sl][ai], 0, 0, 0);
                }
            }
        }
    }
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
        const int ti = wave + 4 * sl;
        if (ti >= ntiles) break;
        const int bt = ti / tiles_c, ct = ti % tiles_c;
#pragma unroll
        for (int ai = 0; ai < NA; ++ai) {
            // accumulator: lane x = column c, register v = row b' = 8 (v / 4) + 4 h + v % 4
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int bp = 32 * bt + 8 * (v / 4) + 4 * h + (v % 4);
                su[L.zv + ((size_t)(a0 + ai) * mcols + bp) * dv + 32 * ct + x] += acc[sl][ai][v];
            }
            if (ct == 0) {                                 // the "ones" column: lanes x = row b', both halves
                const float tot = drow[sl][ai] + __shfl_xor(drow[sl][ai], 32);
                if (h == 0) su[L.zd + (size_t)(a0 + ai) * mcols + 32 * bt + x] += tot;
            }
        }
    }
}

template <typename T>
psf_status step_launch(const Problem &pb, const void *q, const void *k, const void *v, const void *G, int pos,
                       float *state, void *o, hipStream_t s)
{
    const DecodeLayout L = decode_layout(pb);
    const int slot = pos % pb.b, le = pb.local_exact ? 1 : 0;
    // sketches of the new token: the general sketch kernel on [units, 1, d]
    Problem one = pb;
    one.n = 1;
    psf_status st = general_sketch_pair_f32(one, q, k, G, state + L.mq, state + L.mk, s);   // one launch for both
    if (st != PSF_OK) return st;
    const int have_state = pos >= pb.b ? 1 : 0;          // Z is zero during the first block
    hipLaunchKernelGGL(dec_state_kernel<T>, dim3(kSlices, (unsigned)pb.units), dim3(kThreads), 0, s, (const T *)q,
                       state, state + L.mq, state + L.part, L, pb.d, pb.dv, pb.p, pb.mcols, pb.F, slot, have_state, le);
    PSF_LAUNCH_CHECK();
    hipLaunchKernelGGL(dec_finish_kernel<T>, dim3((unsigned)pb.units), dim3(kThreads), 0, s, (const T *)q,
                       (const T *)k, (const T *)v, state, state + L.mq, state + L.mk, state + L.part, (T *)o, L, pb.d,
                       pb.dv, pb.p, pb.mcols, slot, le);
    PSF_LAUNCH_CHECK();
    if (slot == pb.b - 1) {                               // the block is complete: fold it into Z
        const dim3 fgrid((unsigned)((pb.F + kFoldFeat - 1) / kFoldFeat), (unsigned)pb.units);
        if (pb.bf16 && pb.mcols % 32 == 0 && pb.mcols <= kFoldMfmaMaxM && pb.dv % 32 == 0 && pb.dv <= kFoldMfmaMaxDv) {
            if ((pb.mcols / 32) * (pb.dv / 32) <= 4)        // one tile per wave: eight sketch rows per workgroup
                hipLaunchKernelGGL(dec_fold_mfma_kernel<1>, dim3((unsigned)pb.mcols / 8, (unsigned)pb.units),
                                   dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols);
            else                                            // two tiles per wave: four rows
                hipLaunchKernelGGL(dec_fold_mfma_kernel<2>, dim3((unsigned)pb.mcols / 4, (unsigned)pb.units),
                                   dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols);
        } else if (pb.dv <= 32)
            hipLaunchKernelGGL((dec_fold_kernel<T, 8>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, pb.F);
        else if (pb.dv <= 64)
            hipLaunchKernelGGL((dec_fold_kernel<T, 16>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, pb.F);
        else if (pb.dv <= 128)
            hipLaunchKernelGGL((dec_fold_kernel<T, 32>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, pb.F);
        else
            hipLaunchKernelGGL((dec_fold_kernel<T, 64>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, pb.F);
        PSF_LAUNCH_CHECK();
    }
    return PSF_OK;
}

}  // namespace

bool decode_supported(const Problem &pb) { return !pb.exact_feat; }

size_t decode_state_bytes(const Problem &pb) { return decode_layout(pb).total * sizeof(float); }

psf_status decode_reset(const Problem &pb, void *state, hipStream_t s)
{
    const size_t count = decode_layout(pb).total;
    hipLaunchKernelGGL(dec_zero_kernel, dim3(2048), dim3(kThreads), 0, s, (float *)state, count);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}

psf_status decode_step(const Problem &pb, const void *q, const void *k, const void *v, const void *G, int pos,
                       void *state, void *o, hipStream_t s)
{
    return pb.bf16 ? step_launch<bf16_t>(pb, q, k, v, G, pos, (float *)state, o, s)
                   : step_launch<float>(pb, q, k, v, G, pos, (float *)state, o, s);
}

}  // namespace psf
