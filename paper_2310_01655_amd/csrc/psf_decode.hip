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
// phi'(x) = m(x) (x) m(x) is symmetric in its two indices, so Z[a][b'] = Z[b'][a] and only the
// pairs a <= b' are kept, the off-diagonal ones doubled: S[a, b'] = Z[a][b'] + Z[b'][a] (b' > a),
// S[a, a] = Z[a][a]; then phi'(q)^T Z = sum_{a <= b'} m(q)[a] m(q)[b'] S[a, b'] -- the same
// numbers from Fs = mcols (mcols + 1) / 2 rows instead of mcols^2.  Pair (a, b') is row
// tri_row(a) + b' - a.
//
// State per (batch, head) unit, caller-owned:
//   ZV [Fs][dv] and ZD [Fs] in fp32: the value columns and the "ones" column of S, kept apart
//   so that rows of ZV are aligned and a step streams them with full-width loads;
//   for bf16 storage also ZH [Fs][dv], ZV rounded to bf16 at every fold: the steps read ZH;
//   then the current block's cache: CK [b][d] keys and CV [b][dv] values in the storage type
//   of the call (fp32 or bf16), CM [b][mcols] sketches m(k) in fp32.
// After the units come the scratch areas: m(q), m(k) of the new token [units][mcols] each and
// the partial sums of the state product [units][kSlices][dv + 1] (used when a unit's product is
// split over several workgroups).
// A step is bound by reading the state once (Fs * (dv * s + 4) bytes per unit, s = 2 with the
// bf16 copy, 4 without) and the cached keys and values of the current block.
#include <type_traits>

#include "psf_internal.h"

namespace psf {
namespace {

constexpr int kThreads = 256;
constexpr int kSlices = 16;        // workgroups per unit in the state product (at most)
constexpr int kMaxPairsPerSlice = 4096;
static_assert((size_t)PSF_MAX_DIM * (PSF_MAX_DIM + 1) / 2 <= (size_t)kSlices * kMaxPairsPerSlice,
              "the largest state fits kSlices slices");

struct DecodeLayout {
    size_t zv, zd, zh, ck, cv, cm, per_unit; // float offsets inside one unit, floats per unit
    size_t mq, mk, part, total;              // float offsets of the scratch areas, total floats
    int shadow;                              // ZH present (see has_shadow)
    int slices;                              // workgroups per unit in the state product
};

// bf16 storage: the steps read a bf16 copy ZH of ZV (rounded once per fold from the fp32 master,
// as the forward kernels round their prefix states), half the bytes of a step.
bool has_shadow(const Problem &pb) { return pb.bf16 && pb.dv % 8 == 0 && pb.dv / 8 <= kThreads; }

// first row of the pairs (a, b' >= a) in the packed upper triangle of an m x m grid
__host__ __device__ inline long long tri_row(int a, int m) { return (long long)a * m - (long long)a * (a - 1) / 2; }
__host__ __device__ inline long long tri_count(int m) { return (long long)m * (m + 1) / 2; }

// the pair of packed row t: a = the largest row index with tri_row(a) <= t (closed form in
// fp32, then corrected by steps of one)
__device__ __forceinline__ void tri_pair(long long t, int m, int &a, int &bp)
{
    const float s = 2.f * m + 1.f;
    int aa = (int)((s - sqrtf(fmaxf(s * s - 8.f * (float)t, 0.f))) * 0.5f);
    aa = max(0, min(aa, m - 1));
    while (aa > 0 && tri_row(aa, m) > t) --aa;
    while (aa + 1 < m && tri_row(aa + 1, m) <= t) ++aa;
    a = aa;
    bp = aa + (int)(t - tri_row(aa, m));
}

DecodeLayout decode_layout(const Problem &pb)
{
    DecodeLayout L;
    auto up = [](size_t v) { return (v + 63) / 64 * 64; };            // 256-byte pieces
    const size_t Fs = (size_t)tri_count(pb.mcols);
    L.shadow = has_shadow(pb) ? 1 : 0;
    // rows per slice: enough for every thread to keep eight 16-byte loads in flight
    // A workgroup costs about a microsecond to start and wind up, as much as streaming a few
    // hundred kilobytes: as few slices as still give every CU about three workgroups, each
    // with at least 256 rows (eight 16-byte loads in flight per thread).
    // A slice's products m(q)[a] m(q)[b'] sit in LDS: at most kMaxPairsPerSlice of them.
    const size_t want = (768 + (size_t)pb.units - 1) / (size_t)pb.units, most = Fs / 256 > 0 ? Fs / 256 : 1;
    const size_t least = (Fs + kMaxPairsPerSlice - 1) / kMaxPairsPerSlice;
    L.slices = (int)(want < most ? want : most);
    if (L.slices < (int)least) L.slices = (int)least;
    if (L.slices > kSlices) L.slices = kSlices;
    L.zv = 0;
    L.zd = up(Fs * pb.dv);
    L.zh = L.zd + up(Fs);
    const size_t per_float = pb.bf16 ? 2 : 1;                         // cached keys / values keep the storage type
    L.ck = L.zh + up(L.shadow ? (Fs * pb.dv + 1) / 2 : 0);
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

// sixteen bytes of a state row as floats: four fp32 or eight bf16 columns
template <typename ZT> struct ZRow;
template <> struct ZRow<float> {
    static constexpr int NV = 4;
    float4 raw;
    __device__ __forceinline__ void load(const float *p) { raw = *(const float4 *)p; }
    __device__ __forceinline__ void zero() { raw = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void fma(float ph, float *acc) const
    {
        acc[0] += ph * raw.x; acc[1] += ph * raw.y; acc[2] += ph * raw.z; acc[3] += ph * raw.w;
    }
    __device__ __forceinline__ float dot(const float *q) const
    {
        return q[0] * raw.x + q[1] * raw.y + q[2] * raw.z + q[3] * raw.w;
    }
};
template <> struct ZRow<bf16_t> {
    static constexpr int NV = 8;
    uint4 raw;
    __device__ __forceinline__ void load(const bf16_t *p) { raw = *(const uint4 *)p; }
    __device__ __forceinline__ void zero() { raw = make_uint4(0u, 0u, 0u, 0u); }
    __device__ __forceinline__ void fma(float ph, float *acc) const
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[2 * i] += ph * __uint_as_float(w[i] << 16);
            acc[2 * i + 1] += ph * __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ __forceinline__ float dot(const float *q) const
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
        float sacc = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            sacc += q[2 * i] * __uint_as_float(w[i] << 16) + q[2 * i + 1] * __uint_as_float(w[i] & 0xffff0000u);
        return sacc;
    }
};

// sum of 256 floats in LDS by the first wave (call with every thread; result valid for tid 0)
__device__ __forceinline__ float sum256(const float *red)
{
    const int tid = threadIdx.x;
    float v = 0.f;
    if (tid < 64) {
        v = (red[tid] + red[tid + 64]) + (red[tid + 128] + red[tid + 192]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    }
    return v;
}

// Sum over the nf rows of z [nf][dv] of phi[row] * z[row][.] into rowp[0 .. dv): NV columns per
// thread (16-byte loads), consecutive lane groups on consecutive rows so that a wave reads
// contiguous kilobytes, eight rows in flight per thread.  issue() starts the loads of the
// first eight rows of every thread -- they do not depend on the query, so the kernel calls it
// before anything else -- and finish() multiplies and goes on with the remaining rows.
// `scratch` (NV * kThreads floats) may alias phi: it is written only after every thread has
// finished reading phi.
template <typename ZT>
struct StateRows {
    static constexpr int NV = ZRow<ZT>::NV;
    const ZT *zc;
    int nf, dv, cp, grp, g;
    bool active, lane_on;
    ZRow<ZT> first[8];

    __device__ __forceinline__ void issue(const ZT *z, int nf_, int dv_)
    {
        const int tid = threadIdx.x, cn = dv_ / NV;
        nf = nf_;
        dv = dv_;
        cp = 1;
        while (cp < cn) cp *= 2;
        grp = kThreads / cp;
        g = tid / cp;
        lane_on = tid % cp < cn;
        zc = z + (tid % cp) * NV;
        active = true;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            first[i].zero();
            if (lane_on && g + i * grp < nf) first[i].load(zc + (size_t)(g + i * grp) * dv);
        }
    }

    __device__ __forceinline__ void finish(const float *phi, float *scratch, float *rowp)
    {
        const int tid = threadIdx.x;
        float s0[NV], s1[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) s0[j] = s1[j] = 0.f;
        if (lane_on) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (g + i * grp < nf) first[i].fma(phi[g + i * grp], (i & 1) ? s1 : s0);
            int ff = g + 8 * grp;
            for (; ff + 7 * grp < nf; ff += 8 * grp) {
                ZRow<ZT> zr[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) zr[i].load(zc + (size_t)(ff + i * grp) * dv);
#pragma unroll
                for (int i = 0; i < 8; ++i) zr[i].fma(phi[ff + i * grp], (i & 1) ? s1 : s0);
            }
            for (; ff < nf; ff += grp) {
                ZRow<ZT> zr;
                zr.load(zc + (size_t)ff * dv);
                zr.fma(phi[ff], s0);
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NV; ++j) scratch[NV * tid + j] = s0[j] + s1[j];
        __syncthreads();
        if (tid < dv) {
            const int cc = tid / NV, j = tid % NV;
            float sacc = 0.f;
            for (int q2 = 0; q2 < grp; ++q2) sacc += scratch[NV * (q2 * cp + cc) + j];
            rowp[tid] = sacc;
        }
    }
};

// In-block share of a slice: rowp[0 .. dv) += sum_j w_j v_j and rowp[dv] += sum_j w_j over the
// cached tokens j_beg .. j_end - 1, w_j = <qs, key_j>^pw.  A group of `lg` neighbouring lanes
// owns a cached row: lane li reads sixteen bytes of the key row, the group adds up the dot
// product with shuffles, and the same lane then weighs sixteen bytes of the value row -- no
// LDS between the two; four rows in flight per thread, the first four started by issue()
// before the query is known.  Needs wa % NK == 0, dv % NV == 0 and lg <= 64 (see
// cache_rows_group).
template <typename KT, typename VT>
struct CacheRows {
    static constexpr int NK = ZRow<KT>::NV, NV = ZRow<VT>::NV, U = 4;
    const KT *keys;
    const VT *vals;
    int wa, dv, j_beg, j_end, lg, li, g, rows_per_pass;
    ZRow<KT> k_first[U];
    ZRow<VT> v_first[U];

    __device__ __forceinline__ void load_rows(int j0, ZRow<KT> *kr, ZRow<VT> *vr) const
    {
#pragma unroll
        for (int i = 0; i < U; ++i) {
            const int row = j0 + i * rows_per_pass + g;
            kr[i].zero();
            vr[i].zero();
            if (row < j_end && li < wa / NK) kr[i].load(keys + (size_t)row * wa + li * NK);
            if (row < j_end && li < dv / NV) vr[i].load(vals + (size_t)row * dv + li * NV);
        }
    }

    __device__ __forceinline__ void issue(const KT *keys_, int wa_, const VT *vals_, int dv_, int j_beg_,
                                          int j_end_, int lg_)
    {
        const int tid = threadIdx.x;
        keys = keys_; vals = vals_; wa = wa_; dv = dv_; j_beg = j_beg_; j_end = j_end_; lg = lg_;
        li = tid % lg;
        g = tid / lg;
        rows_per_pass = kThreads / lg;
        load_rows(j_beg, k_first, v_first);
    }

    __device__ __forceinline__ void finish(const float *qs, int pw, float *scratch, float *red, float *rowp)
    {
        const int tid = threadIdx.x;
        float qreg[NK];
#pragma unroll
        for (int j = 0; j < NK; ++j) qreg[j] = li < wa / NK ? qs[li * NK + j] : 0.f;
        float acc[NV], wsum = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) acc[j] = 0.f;
        auto weigh = [&](int j0, const ZRow<KT> *kr, const ZRow<VT> *vr) {
#pragma unroll
            for (int i = 0; i < U; ++i) {
                float sdot = kr[i].dot(qreg);
                for (int off = 1; off < lg; off *= 2) sdot += __shfl_xor(sdot, off);
                float wv = 1.f;
                for (int e = 0; e < pw; ++e) wv *= sdot;
                if (j0 + i * rows_per_pass + g >= j_end) wv = 0.f;
                vr[i].fma(wv, acc);
                if (li == 0) wsum += wv;
            }
        };
        weigh(j_beg, k_first, v_first);
        // uniform bounds: every lane takes part in the shuffles
        for (int j0 = j_beg + U * rows_per_pass; j0 < j_end; j0 += U * rows_per_pass) {
            ZRow<KT> kr[U];
            ZRow<VT> vr[U];
            load_rows(j0, kr, vr);
            weigh(j0, kr, vr);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NV; ++j) scratch[NV * tid + j] = acc[j];
        red[tid] = wsum;
        __syncthreads();
        if (tid < dv) {
            const int cc = tid / NV, j = tid % NV;
            float sacc = 0.f;
            for (int q2 = 0; q2 < rows_per_pass; ++q2) sacc += scratch[NV * (q2 * lg + cc) + j];
            rowp[tid] += sacc;
        }
        const float tot = sum256(red);
        if (tid == 0) rowp[dv] += tot;
    }
};

// lane-group size for CacheRows, or 0 when the shapes do not fit it
__device__ __forceinline__ int cache_rows_group(int wa, int nk, int dv, int nv)
{
    if (wa % nk != 0 || dv % nv != 0) return 0;
    int lg = 1;
    while (lg < wa / nk || lg < dv / nv) lg *= 2;
    return lg <= 64 ? lg : 0;
}

__global__ __launch_bounds__(kThreads) void dec_zero_kernel(float *__restrict__ p, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += (size_t)gridDim.x * kThreads)
        p[i] = 0.f;
}

// part[u][s][c] = the share of slice s in row [N | S] of the new token:
//   cross-block: sum over the packed pairs f = (a, b') of the slice of m(q)[a] m(q)[b'] ZV[f][c]
//   (c < dv; read from the bf16 copy when SHADOW) and, at c = dv, of the same times ZD[f] (only
//   once a block is complete: have_state; F = the number of pairs); the products of the slice
//   sit in LDS;
//   in-block: the slice's share of the `slot` tokens cached since the last block boundary,
//   sum_j w_j [v_j | 1] with the weights of Section 3.2 (LE: keys in the storage type) or 3.1
//   (their fp32 sketches).  The new token itself is not in the cache yet: its own pair is added
//   by dec_finish_kernel.
// The first loads of both parts are issued before the query is read, so that a workgroup waits
// for memory once and not four times in a row.
// MODE 0: slices; dec_finish_kernel adds them up.  MODE 1 (one slice per unit): the workgroup
// has the whole row, so it also does what dec_finish_kernel does -- the new token's own pair,
// the division, the cache append.  MODE 2: it also computes m(q) and m(k) of the new token
// itself (Algorithm 1 with the matrices of the unit's head), and the step is one launch.
// MODE 3: slices as in MODE 0, but every slice sketches the token itself (slice 0 leaves the
// sketches in mq_out / mk_out for dec_finish_kernel): two launches instead of three.
struct DecSketchArgs {
    const void *G;           // sketch matrices, storage type
    size_t g_len;            // entries per set
    int heads, per_head, r;
};

template <typename T, bool SHADOW, bool LE, int MODE>
__global__ __launch_bounds__(kThreads) void dec_state_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                             const T *__restrict__ v, float *__restrict__ state,
                                                             const float *__restrict__ mq_new,
                                                             const float *__restrict__ mk_new,
                                                             float *__restrict__ mq_out, float *__restrict__ mk_out,
                                                             float *__restrict__ part, T *__restrict__ o,
                                                             DecodeLayout L, int d, int dv, int p, int mcols,
                                                             long long F, int slot, int have_state,
                                                             DecSketchArgs sk)
{
    constexpr bool FUSE = MODE == 1 || MODE == 2, SK = MODE >= 2;
    static_assert(kThreads == kSketchThreads, "sketch_row_lds assumes this workgroup size");
    using ZT = std::conditional_t<SHADOW, bf16_t, float>;
    using KT = std::conditional_t<LE, T, float>;
    constexpr int kMaxPer = kMaxPairsPerSlice;             // decode_layout keeps a slice within this
    __shared__ float mq[PSF_MAX_DIM], qs[PSF_MAX_DIM], red[kThreads], w[kThreads], rowp[PSF_MAX_DIM + 1];
    __shared__ float xk[SK ? PSF_MAX_DIM : 1], mk_s[SK ? PSF_MAX_DIM : 1], xq[SK && !LE ? PSF_MAX_DIM : 1];
    __shared__ union {
        float phi[kMaxPer];          // products of the slice; later the scratch of the reductions
        SketchScratchN<2> sketch;    // before that (MODE 2): intermediates of Algorithm 1 for q and k
    } big;
    float *const phi = big.phi;
    const int u = blockIdx.y, sl = blockIdx.x, tid = threadIdx.x, kc = dv + 1;
    float *su = state + (size_t)u * L.per_unit;
    const int wa = LE ? d : mcols, slices = L.slices;
    // this slice's pairs and cached tokens
    const long long per = (F + slices - 1) / slices;
    const long long f_beg = sl * per;
    const int nf = have_state ? (int)max(0LL, min(F, f_beg + per) - f_beg) : 0;
    const int per_j = (slot + slices - 1) / slices;
    const int j_beg = min(slot, sl * per_j), j_end = min(slot, j_beg + per_j);
    const float *zv = su + L.zv + (size_t)f_beg * dv;
    const float *zd = su + L.zd + f_beg;
    const ZT *zrows = SHADOW ? (const ZT *)((const bf16_t *)(su + L.zh) + (size_t)f_beg * dv) : (const ZT *)zv;
    const KT *keys = LE ? (const KT *)(su + L.ck) : (const KT *)(su + L.cm);
    const T *cvals = (const T *)(su + L.cv);
    const bool zfast = dv % ZRow<ZT>::NV == 0 && dv / ZRow<ZT>::NV <= kThreads;
    const int lg = cache_rows_group(wa, ZRow<KT>::NV, dv, ZRow<T>::NV);

    // every load that does not depend on another one, oldest first (loads complete in order):
    // the query (mcols, wa <= 256: one element per thread), the ones column, the first state
    // rows, the first cached rows
    static_assert(PSF_MAX_DIM <= kThreads, "one query element per thread");
    float mq_reg = 0.f, qs_reg = 0.f, xq_reg = 0.f, xk_reg = 0.f;
    if constexpr (SK) {
        if (tid < d) {
            xq_reg = load_f(q, (size_t)u * d + tid);
            xk_reg = load_f(k, (size_t)u * d + tid);
        }
    } else {
        if (tid < mcols) mq_reg = mq_new[(size_t)u * mcols + tid];
        if (tid < wa) qs_reg = LE ? load_f(q, (size_t)u * d + tid) : mq_new[(size_t)u * mcols + tid];
    }
    const float zd0 = tid < nf ? zd[tid] : 0.f, zd1 = tid + kThreads < nf ? zd[tid + kThreads] : 0.f;
    StateRows<ZT> sr;
    CacheRows<KT, T> cr;
    if (zfast && nf > 0) sr.issue(zrows, nf, dv);
    if (lg > 0 && j_end > j_beg) cr.issue(keys, wa, cvals, dv, j_beg, j_end, lg);

    for (int c = tid; c < kc; c += kThreads) rowp[c] = 0.f;
    if constexpr (SK) {
        // raw rows into LDS (q in qs when the in-block weights use it, else in xq), then
        // Algorithm 1 for q and k together; the results leave the scratch before it is reused
        float *const xq_s = LE ? qs : xq;
        if (tid < d) {
            xq_s[tid] = xq_reg;
            xk[tid] = xk_reg;
        }
        __syncthreads();
        const T *g_set = (const T *)sk.G + (sk.per_head ? (size_t)(u % sk.heads) * sk.g_len : 0);
        const float *const rows[2] = {xq_s, xk};
        const float *fin[2];
        sketch_rows_lds<T, 2>(rows, g_set, d, sk.r, p, big.sketch, fin);
        if (tid < mcols) {
            mq[tid] = fin[0][tid];
            if (!LE) qs[tid] = fin[0][tid];
            mk_s[tid] = fin[1][tid];
            if constexpr (MODE == 3) {
                if (sl == 0) {                             // for dec_finish_kernel
                    mq_out[(size_t)u * mcols + tid] = fin[0][tid];
                    mk_out[(size_t)u * mcols + tid] = fin[1][tid];
                }
            }
        }
    } else {
        if (tid < mcols) mq[tid] = mq_reg;
        if (tid < wa) qs[tid] = qs_reg;
    }
    __syncthreads();
    const int dvp = pow2_at_least(dv, 32, kThreads), groups = kThreads / dvp;
    float *out = part + ((size_t)u * kSlices + sl) * kc;

    if (nf > 0) {
        for (int ff = tid; ff < nf; ff += kThreads) {
            int a, bp;
            tri_pair(f_beg + ff, mcols, a, bp);
            phi[ff] = mq[a] * mq[bp];
        }
        __syncthreads();
        // the ones column first: it reads phi, which StateRows::finish then reuses as scratch
        float a1c = 0.f;
        if (tid < nf) a1c = phi[tid] * zd0;
        if (tid + kThreads < nf) a1c += phi[tid + kThreads] * zd1;
        for (int ff = tid + 2 * kThreads; ff < nf; ff += kThreads) a1c += phi[ff] * zd[ff];
        red[tid] = a1c;
        if (zfast) {
            sr.finish(phi, phi, rowp);
        } else {
            for (int c0 = 0; c0 < dv; c0 += dvp) {
                const int c = c0 + tid % dvp, g = tid / dvp;
                float a0 = 0.f;
                if (c < dv)
                    for (int ff = g; ff < nf; ff += groups) a0 += phi[ff] * zv[(size_t)ff * dv + c];
                __syncthreads();
                w[tid] = a0;
                __syncthreads();
                if (tid < dvp && c0 + tid < dv) {
                    float sacc = 0.f;
                    for (int q2 = 0; q2 < groups; ++q2) sacc += w[q2 * dvp + tid];
                    rowp[c0 + tid] = sacc;
                }
            }
        }
        __syncthreads();                                    // red complete in either branch
        const float tot = sum256(red);
        if (tid == 0) rowp[dv] = tot;
    }

    // in-block: cached tokens j_beg .. j_end - 1 of this slice
    if (lg > 0) {
        if (j_end > j_beg) {
            __syncthreads();                               // phi (the scratch below) and red are free
            cr.finish(qs, LE ? p : 2, phi, red, rowp);
        }
    } else {
        for (int j0 = j_beg; j0 < j_end; j0 += kThreads) {
            const int nj = min(kThreads, j_end - j0);
            __syncthreads();
            // weights of the pass: four threads per key, 64 keys at a time
            for (int kk = 0; kk < nj; kk += kThreads / 4) {
                const int kj = kk + (tid >> 2), part4 = tid & 3;
                float sdot = 0.f;
                if (kj < nj) {
                    const size_t roff = (size_t)(j0 + kj) * wa;
                    for (int e = part4; e < wa; e += 4) sdot += qs[e] * load_f(keys, roff + e);
                }
                sdot += __shfl_xor(sdot, 1);
                sdot += __shfl_xor(sdot, 2);
                if (part4 == 0 && kj < nj) {
                    float wv = sdot * sdot;
                    if (LE) {
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
    }
    __syncthreads();
    if constexpr (!FUSE) {
        for (int c = tid; c < kc; c += kThreads) out[c] = rowp[c];
    } else {
        // own pair <q, k>^p (or <m(q), m(k)>^2), then N / (1 + S) and the cache append
        float k_own = 0.f;
        if constexpr (SK) {
            if (tid < wa) k_own = LE ? xk[tid] : mk_s[tid];
        } else {
            if (tid < wa) k_own = LE ? load_f(k, (size_t)u * d + tid) : mk_new[(size_t)u * mcols + tid];
        }
        red[tid] = tid < wa ? qs[tid] * k_own : 0.f;
        __syncthreads();
        const float sdot = sum256(red);
        if (tid == 0) {
            float wv = 1.f;
            for (int e = 0; e < (LE ? p : 2); ++e) wv *= sdot;
            w[0] = wv;
        }
        __syncthreads();
        const float w_self = w[0], den = 1.f + rowp[dv] + w_self;
        T *ckeys = (T *)(su + L.ck), *cv_out = (T *)(su + L.cv);
        for (int c = tid; c < dv; c += kThreads) {
            const T vraw = v[(size_t)u * dv + c];
            store_f(o, (size_t)u * dv + c, (rowp[c] + w_self * load_f(&vraw, 0)) / den);
            cv_out[(size_t)slot * dv + c] = vraw;
        }
        for (int e = tid; e < d; e += kThreads) ckeys[(size_t)slot * d + e] = k[(size_t)u * d + e];
        for (int e = tid; e < mcols; e += kThreads)
            su[L.cm + (size_t)slot * mcols + e] = SK ? mk_s[e] : mk_new[(size_t)u * mcols + e];
    }
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
    for (int sidx = 0; sidx < L.slices; ++sidx) den += part[((size_t)u * kSlices + sidx) * kc + dv];
    for (int c = tid; c < dv; c += kThreads) {
        float acc = w_self * load_f(v, (size_t)u * dv + c);
        for (int sidx = 0; sidx < L.slices; ++sidx) acc += part[((size_t)u * kSlices + sidx) * kc + c];
        store_f(o, (size_t)u * dv + c, acc / den);
    }
}

// ZV[f][c] += sum over the b cached tokens of w_f m_j[a] m_j[b'] v_j[c] for the packed pair
// f = (a, b'), w_f = 2 off the diagonal and 1 on it; ZD[f] += the same without v.
// Workgroup = kFoldFeat pairs; thread (c, g) owns the PER = kFoldFeat / groups pairs
// g * PER .. of column c (groups = 256 / columns per pass).
constexpr int kFoldFeat = 64, kFoldTok = 32;
template <typename T, int PER>
__global__ __launch_bounds__(kThreads) void dec_fold_kernel(float *__restrict__ state, DecodeLayout L,
                                                            int dv, int b, int mcols, long long F)
{
    __shared__ float phi[kFoldTok][kFoldFeat + 1], vt[kFoldTok][PSF_MAX_DIM], pair_w[kFoldFeat];
    __shared__ int pair_a[kFoldFeat], pair_b[kFoldFeat];
    constexpr int groups = kFoldFeat / PER, dvp = kThreads / groups;
    const int tid = threadIdx.x, u = blockIdx.y;
    const long long f0 = (long long)blockIdx.x * kFoldFeat;
    float *su = state + (size_t)u * L.per_unit;
    if (tid < kFoldFeat) {
        int a = 0, bp = 0;
        if (f0 + tid < F) tri_pair(f0 + tid, mcols, a, bp);
        pair_a[tid] = a;
        pair_b[tid] = bp;
        pair_w[tid] = f0 + tid < F ? (bp > a ? 2.f : 1.f) : 0.f;
    }
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
                if (jj < lim) {
                    const float *m = su + L.cm + (size_t)(j0 + jj) * mcols;
                    v = pair_w[ff] * m[pair_a[ff]] * m[pair_b[ff]];
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
                if (f0 + g * PER + ff < F) {
                    const size_t at = (size_t)(f0 + g * PER + ff) * dv + c;
                    const float znew = su[L.zv + at] + acc[ff];
                    su[L.zv + at] = znew;
                    if (L.shadow) ((bf16_t *)(su + L.zh))[at] = f32_to_bf16(znew);
                }
        }
        if (c0 == 0 && tid < kFoldFeat && f0 + tid < F) su[L.zd + f0 + tid] += dacc;
    }
}

// The same fold on MFMA for bf16 storage (phi'(k) and v as bf16 operands, fp32 accumulation, as
// the forward state kernel does): S[a, b'][c] += w sum_j (m_j[a] m_j[b']) v_j[c] for b' >= a.
// Workgroup = (NA consecutive sketch rows a, unit).  An item is (row a, 32-wide range of b'):
// the fragment m_j[a] m_j[b'] generated for it feeds one MFMA per 32-wide tile of value columns.
// Ranges whose columns b' all lie below the group's first row are skipped; the remaining items
// are dealt evenly to the four waves, a wave's items sharing one range (and with it the
// fragments of m_j[b'] and of v).  64 tokens at a time are staged transposed ([column][token])
// so that a lane's eight tokens of one column are neighbours.
typedef __bf16 dec_bf16x8 __attribute__((ext_vector_type(8)));
typedef float dec_f32x16 __attribute__((ext_vector_type(16)));
constexpr int kFoldMfmaTok = 64, kFoldMfmaMaxM = 64, kFoldMfmaMaxDv = 128;

template <int MC, int DV>
struct FoldShape {
    static constexpr int NB = MC / 32, TC = DV / 32;
    static constexpr int IPW = 8 / TC < 4 ? 8 / TC : 4;      // items per wave, at most (accumulators: IPW * TC tiles)
    static constexpr int NA = 4 * IPW / NB;                  // sketch rows per workgroup
};

template <int MC, int DV>
__global__ __launch_bounds__(kThreads, 2) void dec_fold_mfma_kernel(float *__restrict__ state, DecodeLayout L, int b)
{
    constexpr int mcols = MC, dv = DV;
    constexpr int NB = FoldShape<MC, DV>::NB, TC = FoldShape<MC, DV>::TC, IPW = FoldShape<MC, DV>::IPW;
    constexpr int NA = FoldShape<MC, DV>::NA;
    // rows of 64 tokens: pitches of 68 floats / 72 bf16 keep every 16-byte read aligned and spread
    // the 16 lanes of a read phase over all banks
    constexpr int TOK = kFoldMfmaTok, PITCH = TOK + 4, PITCHV = TOK + 8;
    __shared__ __attribute__((aligned(16))) float mts[MC][PITCH];
    __shared__ __attribute__((aligned(16))) bf16_t vts[DV][PITCHV];
    // The MC / NA workgroups of a unit all stream the unit's block cache.  Consecutive workgroup
    // ids go to different XCDs, so give each XCD a contiguous range of (unit, row group) pairs:
    // the groups of a unit then share one L2 and run at about the same time.
    constexpr int GROUPS = MC / NA;
    int wg = blockIdx.x;
    if ((gridDim.x & 7) == 0) wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int u = wg / GROUPS, a0 = (wg % GROUPS) * NA;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 31, h = lane >> 5;
    float *su = state + (size_t)u * L.per_unit;
    // this wave's items: rows a0 + row0 .. + rpw - 1 of range bt
    const int bt_min = a0 / 32, nb_act = NB - bt_min;
    const int rpw = NA * nb_act / 4;                         // 1 .. IPW
    const int bt = bt_min + (wave * rpw) / NA, row0 = (wave * rpw) % NA;
    dec_f32x16 acc[IPW][TC];
    float drow[IPW];
#pragma unroll
    for (int k = 0; k < IPW; ++k) {
        drow[k] = 0.f;
#pragma unroll
        for (int ct = 0; ct < TC; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[k][ct][v] = 0.f;
    }
    // A chunk of 64 tokens goes global -> registers (16-byte / 8-byte pieces of a cached row) ->
    // LDS (transposed); the loads of the next chunk are in flight while this one is multiplied.
    constexpr int MP = TOK * MC / 4 / kThreads, VP = TOK * DV / 4 / kThreads;
    float4 m_pre[MP];
    uint2 v_pre[VP];
    const float *cm = su + L.cm;
    const bf16_t *cvv = (const bf16_t *)(su + L.cv);
    auto fetch = [&](int j0) {
#pragma unroll
        for (int i = 0; i < MP; ++i) {
            const int idx = tid + i * kThreads, jj = idx / (MC / 4), c4 = idx % (MC / 4);
            m_pre[i] = j0 + jj < b ? *(const float4 *)(cm + (size_t)(j0 + jj) * MC + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int idx = tid + i * kThreads, jj = idx / (DV / 4), c4 = idx % (DV / 4);
            v_pre[i] = j0 + jj < b ? *(const uint2 *)(cvv + (size_t)(j0 + jj) * DV + 4 * c4) : make_uint2(0u, 0u);
        }
    };
    auto put = [&]() {
#pragma unroll
        for (int i = 0; i < MP; ++i) {
            const int idx = tid + i * kThreads, jj = idx / (MC / 4), c4 = idx % (MC / 4);
            mts[4 * c4 + 0][jj] = m_pre[i].x; mts[4 * c4 + 1][jj] = m_pre[i].y;
            mts[4 * c4 + 2][jj] = m_pre[i].z; mts[4 * c4 + 3][jj] = m_pre[i].w;
        }
#pragma unroll
        for (int i = 0; i < VP; ++i) {
            const int idx = tid + i * kThreads, jj = idx / (DV / 4), c4 = idx % (DV / 4);
            vts[4 * c4 + 0][jj] = (bf16_t)(v_pre[i].x & 0xffffu); vts[4 * c4 + 1][jj] = (bf16_t)(v_pre[i].x >> 16);
            vts[4 * c4 + 2][jj] = (bf16_t)(v_pre[i].y & 0xffffu); vts[4 * c4 + 3][jj] = (bf16_t)(v_pre[i].y >> 16);
        }
    };
    fetch(0);
    for (int j0 = 0; j0 < b; j0 += TOK) {
        __syncthreads();
        put();
        __syncthreads();
        if (j0 + TOK < b) fetch(j0 + TOK);
#pragma unroll
        for (int sstep = 0; sstep < TOK / 16; ++sstep) {
            const int tok = 16 * sstep + 8 * h;
            const float4 mb0 = *(const float4 *)&mts[32 * bt + x][tok], mb1 = *(const float4 *)&mts[32 * bt + x][tok + 4];
            const float mb[8] = {mb0.x, mb0.y, mb0.z, mb0.w, mb1.x, mb1.y, mb1.z, mb1.w};
            dec_bf16x8 fb[TC];
#pragma unroll
            for (int ct = 0; ct < TC; ++ct) fb[ct] = *(const dec_bf16x8 *)&vts[32 * ct + x][tok];
#pragma unroll
            for (int k = 0; k < IPW; ++k) {
                if (k >= rpw) break;                        // wave-uniform
                const int a = a0 + row0 + k;
                const float4 ma0 = *(const float4 *)&mts[a][tok], ma1 = *(const float4 *)&mts[a][tok + 4];
                const float ma[8] = {ma0.x, ma0.y, ma0.z, ma0.w, ma1.x, ma1.y, ma1.z, ma1.w};
                dec_bf16x8 fa;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float pr = ma[e] * mb[e];
                    fa[e] = (__bf16)pr;
                    drow[k] += pr;
                }
#pragma unroll
                for (int ct = 0; ct < TC; ++ct)
                    acc[k][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb[ct], acc[k][ct], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < IPW; ++k) {
        if (k >= rpw) break;
        const int a = a0 + row0 + k;
        const size_t rowbase = (size_t)tri_row(a, mcols);
#pragma unroll
        for (int ct = 0; ct < TC; ++ct) {
            // accumulator: lane x = column c, register v = row b' = 8 (v / 4) + 4 h + v % 4
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int bp = 32 * bt + 8 * (v / 4) + 4 * h + (v % 4);
                if (bp >= a) {
                    const size_t at = (rowbase + bp - a) * dv + 32 * ct + x;
                    const float znew = su[L.zv + at] + (bp > a ? 2.f : 1.f) * acc[k][ct][v];
                    su[L.zv + at] = znew;
                    if (L.shadow) ((bf16_t *)(su + L.zh))[at] = f32_to_bf16(znew);
                }
            }
        }
        // the "ones" column: lanes x = row b', both halves
        const float tot = drow[k] + __shfl_xor(drow[k], 32);
        const int bp = 32 * bt + x;
        if (h == 0 && bp >= a) su[L.zd + rowbase + bp - a] += (bp > a ? 2.f : 1.f) * tot;
    }
}

// Prompt tokens pos0 + j (j < count) of every unit go into cache slots j: keys and values as
// they are, m(k) from Algorithm 1 (two tokens at a time share the matrices) or, HAVE_M, from
// the rows M_all [units][n_prompt][mcols] computed beforehand (learned sketches).
constexpr int kPrefillTokens = 8;
template <typename T, bool HAVE_M>
__global__ __launch_bounds__(kThreads) void dec_prefill_kernel(const T *__restrict__ K, const T *__restrict__ V,
                                                               const float *__restrict__ M_all,
                                                               float *__restrict__ state, DecodeLayout L, int d,
                                                               int dv, int p, int mcols, int n_prompt, int pos0,
                                                               int count, int m_first, int m_rows, DecSketchArgs sk)
{
    // M_all: [units][m_rows][mcols], the sketches of prompt rows m_first .. m_first + m_rows - 1
    static_assert(kThreads == kSketchThreads, "sketch_rows_lds assumes this workgroup size");
    __shared__ float xs[2][PSF_MAX_DIM];
    __shared__ SketchScratchN<HAVE_M ? 1 : 2> scratch;
    const int u = blockIdx.y, tid = threadIdx.x;
    float *su = state + (size_t)u * L.per_unit;
    T *ckeys = (T *)(su + L.ck), *cvals = (T *)(su + L.cv);
    const T *g_set = (const T *)sk.G + (sk.per_head ? (size_t)(u % sk.heads) * sk.g_len : 0);
    // kPrefillTokens tokens per workgroup, two at a time (a workgroup per pair would spend most
    // of its time starting up)
    for (int j0 = kPrefillTokens * blockIdx.x; j0 < min(count, kPrefillTokens * ((int)blockIdx.x + 1)); j0 += 2) {
        const int nrow = min(2, count - j0);
        for (int i = 0; i < nrow; ++i) {
            const size_t row = (size_t)u * n_prompt + pos0 + j0 + i;
            for (int e = tid; e < d; e += kThreads) ckeys[(size_t)(j0 + i) * d + e] = K[row * d + e];
            for (int c = tid; c < dv; c += kThreads) cvals[(size_t)(j0 + i) * dv + c] = V[row * dv + c];
            if (HAVE_M)
                for (int e = tid; e < mcols; e += kThreads)
                    su[L.cm + (size_t)(j0 + i) * mcols + e] =
                        M_all[((size_t)u * m_rows + (pos0 + j0 + i - m_first)) * mcols + e];
        }
        if constexpr (!HAVE_M) {
            __syncthreads();                               // the previous pair's results have been read
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (tid < d) xs[i][tid] = i < nrow ? load_f(K, ((size_t)u * n_prompt + pos0 + j0 + i) * d + tid) : 0.f;
            __syncthreads();
            const float *const rows[2] = {xs[0], xs[1]};
            const float *fin[2];
            sketch_rows_lds<T, 2>(rows, g_set, d, sk.r, p, scratch, fin);
            for (int i = 0; i < nrow; ++i)
                if (tid < mcols) su[L.cm + (size_t)(j0 + i) * mcols + tid] = fin[i][tid];
        }
    }
}

// The state after the complete blocks of a prompt, taken from the forward path's state kernel:
// Zg [units][a][b'/8][c][8] bf16 holds sum_j phi'(k_j) v_j^T with this file's convention already
// applied (b' > a doubled, b' < a zero); Spart [units][parts][r][r] fp32 the partial m^T m.
// ZV (and its bf16 copy) take the pairs a <= b' of Zg, ZD the weighted sums of the partials.
__global__ __launch_bounds__(kThreads) void dec_import_state_kernel(const bf16_t *__restrict__ Zg,
                                                                    const float *__restrict__ Spart,
                                                                    float *__restrict__ state, DecodeLayout L,
                                                                    int dv, int mcols, long long pairs, int parts)
{
    const int u = blockIdx.y;
    float *su = state + (size_t)u * L.per_unit;
    const bf16_t *zu = Zg + (size_t)u * mcols * mcols * dv;
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    // one 16-byte piece of Zg per thread: row a, eight columns b' = 8 o .., value column c
    // (consecutive threads: consecutive c, so reads and the stores of a row are contiguous)
    if (idx < (long long)mcols * (mcols / 8) * dv) {
        const int c = (int)(idx % dv), o = (int)((idx / dv) % (mcols / 8)), a = (int)(idx / dv / (mcols / 8));
        if (8 * o + 7 >= a) {
            const uint4 raw = *(const uint4 *)(zu + (size_t)idx * 8);
            const uint32_t wds[4] = {raw.x, raw.y, raw.z, raw.w};
            const size_t row0 = (size_t)tri_row(a, mcols);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int bp = 8 * o + e;
                if (bp < a) continue;
                const bf16_t h16 = (bf16_t)((e & 1) ? wds[e / 2] >> 16 : wds[e / 2] & 0xffffu);
                const size_t at = (row0 + bp - a) * dv + c;
                su[L.zv + at] = bf16_to_f32(h16);
                if (L.shadow) ((bf16_t *)(su + L.zh))[at] = h16;
            }
        }
    }
    if (idx < pairs) {
        int a, bp;
        tri_pair(idx, mcols, a, bp);
        const float *sp = Spart + (size_t)u * parts * mcols * mcols + (size_t)a * mcols + bp;
        float sacc = 0.f;
        for (int q2 = 0; q2 < parts; ++q2) sacc += sp[(size_t)q2 * mcols * mcols];
        su[L.zd + idx] = (bp > a ? 2.f : 1.f) * sacc;
    }
}

// 16-byte copies of rows first .. first + rows - 1 of every unit out of [units][n_prompt][w] (bf16)
// into [units][rows][w]
__global__ __launch_bounds__(kThreads) void dec_gather_rows_kernel(const bf16_t *__restrict__ src,
                                                                   bf16_t *__restrict__ dst, int w, int n_prompt,
                                                                   int first, int rows, size_t pieces)
{
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;       // piece of 8 elements
    if (i >= pieces) return;
    const size_t per_unit = (size_t)rows * w / 8;
    const size_t u = i / per_unit, r8 = i % per_unit;
    *(uint4 *)(dst + i * 8) = *(const uint4 *)(src + (u * n_prompt + first) * w + r8 * 8);
}

// Folds the b tokens in the block cache into the state (the block is complete).
template <typename T>
psf_status launch_fold(const Problem &pb, const DecodeLayout &L, float *state, hipStream_t s)
{
    const long long Fs = tri_count(pb.mcols);
    const dim3 fgrid((unsigned)((Fs + kFoldFeat - 1) / kFoldFeat), (unsigned)pb.units);
    if (pb.bf16 && pb.mcols % 32 == 0 && pb.mcols <= kFoldMfmaMaxM && pb.dv % 32 == 0 && pb.dv <= kFoldMfmaMaxDv) {
#define PSF_FOLD(MC_, DV_)                                                                                       \
    if (pb.mcols == MC_ && pb.dv == DV_)                                                                          \
    hipLaunchKernelGGL((dec_fold_mfma_kernel<MC_, DV_>), dim3((unsigned)(MC_ / FoldShape<MC_, DV_>::NA * pb.units)), \
                       dim3(kThreads), 0, s, state, L, pb.b)
        PSF_FOLD(32, 32); PSF_FOLD(32, 64); PSF_FOLD(32, 96); PSF_FOLD(32, 128);
        PSF_FOLD(64, 32); PSF_FOLD(64, 64); PSF_FOLD(64, 96); PSF_FOLD(64, 128);
#undef PSF_FOLD
    } else if (pb.dv <= 32)
        hipLaunchKernelGGL((dec_fold_kernel<T, 8>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, Fs);
    else if (pb.dv <= 64)
        hipLaunchKernelGGL((dec_fold_kernel<T, 16>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, Fs);
    else if (pb.dv <= 128)
        hipLaunchKernelGGL((dec_fold_kernel<T, 32>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, Fs);
    else
        hipLaunchKernelGGL((dec_fold_kernel<T, 64>), fgrid, dim3(kThreads), 0, s, state, L, pb.dv, pb.b, pb.mcols, Fs);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}

template <typename T>
psf_status step_launch(const Problem &pb, const void *q, const void *k, const void *v, const void *G, int pos,
                       float *state, void *o, hipStream_t s)
{
    const DecodeLayout L = decode_layout(pb);
    const int slot = pos % pb.b, le = pb.local_exact ? 1 : 0;
    // one workgroup per unit: it finishes the row itself, and with the sketch of Algorithm 1
    // (no networks) it also sketches the new token
    const bool fuse = L.slices == 1;
    // learned sketches come from the general sketch kernel (modes 0, 1); those of Algorithm 1 are
    // computed inside the step kernel (modes 2, 3)
    const int mode = pb.learned ? (fuse ? 1 : 0) : (fuse ? 2 : 3);
    if (mode < 2) {
        // sketches of the new token: the general sketch kernel on [units, 1, d]
        Problem one = pb;
        one.n = 1;
        psf_status st = general_sketch_pair_f32(one, q, k, G, state + L.mq, state + L.mk, s);   // one launch for both
        if (st != PSF_OK) return st;
    }
    const int have_state = pos >= pb.b ? 1 : 0;          // Z is zero during the first block
    const long long Fs = tri_count(pb.mcols);
    const dim3 sgrid((unsigned)L.slices, (unsigned)pb.units);
    const DecSketchArgs ska{G, pb.g_len, pb.heads, pb.per_head ? 1 : 0, pb.r};
#define PSF_DEC_STATE(SH, LE_, MO)                                                                             \
    hipLaunchKernelGGL((dec_state_kernel<T, SH, LE_, MO>), sgrid, dim3(kThreads), 0, s, (const T *)q,             \
                       (const T *)k, (const T *)v, state, state + L.mq, state + L.mk, state + L.mq, state + L.mk, \
                       state + L.part, (T *)o, L, pb.d, pb.dv, pb.p, pb.mcols, Fs, slot, have_state, ska)
#define PSF_DEC_STATE_MODE(SH, LE_)      \
    do {                                 \
        if (mode == 0)                   \
            PSF_DEC_STATE(SH, LE_, 0);   \
        else if (mode == 1)              \
            PSF_DEC_STATE(SH, LE_, 1);   \
        else if (mode == 2)              \
            PSF_DEC_STATE(SH, LE_, 2);   \
        else                             \
            PSF_DEC_STATE(SH, LE_, 3);   \
    } while (0)
    if (L.shadow) {
        if constexpr (std::is_same_v<T, bf16_t>) {
            if (le) PSF_DEC_STATE_MODE(true, true); else PSF_DEC_STATE_MODE(true, false);
        }
    } else {
        if (le) PSF_DEC_STATE_MODE(false, true); else PSF_DEC_STATE_MODE(false, false);
    }
#undef PSF_DEC_STATE_MODE
#undef PSF_DEC_STATE
    PSF_LAUNCH_CHECK();
    if (!fuse) {                                          // modes 0 and 3: the slices are added up here
        hipLaunchKernelGGL(dec_finish_kernel<T>, dim3((unsigned)pb.units), dim3(kThreads), 0, s, (const T *)q,
                           (const T *)k, (const T *)v, state, state + L.mq, state + L.mk, state + L.part, (T *)o, L,
                           pb.d, pb.dv, pb.p, pb.mcols, slot, le);
        PSF_LAUNCH_CHECK();
    }
    if (slot == pb.b - 1) return launch_fold<T>(pb, L, state, s);   // the block is complete: fold it into Z
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

// The complete blocks of a prompt go through the forward path's kernels where those exist
// (bf16, the MFMA shapes, sketches of Algorithm 1): their total state is imported, and only the
// tokens after the last block boundary are written into the cache one block at a time.
static int prefill_fast_tokens(const Problem &pb, int n_prompt)
{
    const int n_full = n_prompt / pb.b * pb.b;
    return n_full > 0 && pb.mcols % 8 == 0 && mfma_total_state_supported(pb, n_full) ? n_full : 0;
}

// Workspace of a hand-over, in this order: the fp32 sketches of the prompt keys that go through
// the cache (learned sketches only: all of them, or those after the last block boundary when
// the forward kernels take the complete blocks), a contiguous copy of those keys (same case),
// contiguous copies of the complete blocks of K and V (when a tail follows them), the forward
// kernels' own buffers.
struct PrefillPlan {
    int n_full, m_rows;                   // tokens through the forward kernels; sketched rows per unit
    size_t m_bytes, ktail_bytes, copy_bytes, total;
};

static PrefillPlan prefill_plan(const Problem &pb, int n_prompt)
{
    PrefillPlan pl;
    const bool learned = pb.learned && pb.p > 2;
    pl.n_full = prefill_fast_tokens(pb, n_prompt);
    const int tail = n_prompt - pl.n_full;
    pl.m_rows = learned ? tail : 0;
    pl.m_bytes = align_up((size_t)pb.units * pl.m_rows * pb.mcols * sizeof(float), 256);
    pl.ktail_bytes = learned && pl.n_full > 0 ? align_up((size_t)pb.units * tail * pb.d * 2, 256) : 0;
    pl.copy_bytes = pl.n_full > 0 && tail > 0 ? align_up((size_t)pb.units * pl.n_full * pb.d * 2, 256) : 0;
    pl.total = pl.m_bytes + pl.ktail_bytes + 2 * pl.copy_bytes +
               (pl.n_full > 0 ? mfma_total_state_workspace_bytes(pb, pl.n_full) : 0);
    return pl;
}

size_t decode_prefill_workspace_bytes(const Problem &pb, int n_prompt) { return prefill_plan(pb, n_prompt).total; }

bool decode_prefill_uses_mfma(const Problem &pb, int n_prompt) { return prefill_fast_tokens(pb, n_prompt) > 0; }

template <typename T>
static psf_status prefill_launch(const Problem &pb, const void *K, const void *V, const void *G, int n_prompt,
                                 float *state, void *ws, hipStream_t s)
{
    const DecodeLayout L = decode_layout(pb);
    psf_status st = decode_reset(pb, state, s);
    if (st != PSF_OK) return st;
    const PrefillPlan pl = prefill_plan(pb, n_prompt);
    const int first = pl.n_full, tail = n_prompt - first;  // prompt tokens before `first` go through the forward kernels
    float *m_tail = (float *)ws;
    char *ktail = (char *)ws + pl.m_bytes, *wsp = ktail + pl.ktail_bytes;
    if constexpr (std::is_same_v<T, bf16_t>) {
        if (first > 0) {
            const bf16_t *kc = (const bf16_t *)K, *vc = (const bf16_t *)V;
            if (tail > 0) {
                const size_t pieces = (size_t)pb.units * first * pb.d / 8;
                const unsigned grid = (unsigned)((pieces + kThreads - 1) / kThreads);
                hipLaunchKernelGGL(dec_gather_rows_kernel, dim3(grid), dim3(kThreads), 0, s, (const bf16_t *)K,
                                   (bf16_t *)wsp, pb.d, n_prompt, 0, first, pieces);
                PSF_LAUNCH_CHECK();
                hipLaunchKernelGGL(dec_gather_rows_kernel, dim3(grid), dim3(kThreads), 0, s, (const bf16_t *)V,
                                   (bf16_t *)(wsp + pl.copy_bytes), pb.dv, n_prompt, 0, first, pieces);
                PSF_LAUNCH_CHECK();
                kc = (const bf16_t *)wsp;
                vc = (const bf16_t *)(wsp + pl.copy_bytes);
            }
            const void *zg = nullptr;
            const float *spart = nullptr;
            int parts = 0;
            st = mfma_total_state(pb, first, kc, vc, G, wsp + 2 * pl.copy_bytes, s, &zg, &spart, &parts);
            if (st != PSF_OK) return st;
            const long long pairs = tri_count(pb.mcols);
            const long long pieces = (long long)pb.mcols * (pb.mcols / 8) * pb.dv;      // >= pairs
            const dim3 grid((unsigned)((pieces + kThreads - 1) / kThreads), (unsigned)pb.units);
            hipLaunchKernelGGL(dec_import_state_kernel, grid, dim3(kThreads), 0, s, (const bf16_t *)zg, spart, state, L,
                               pb.dv, pb.mcols, pairs, parts);
            PSF_LAUNCH_CHECK();
        }
    }
    const bool have_m = pl.m_rows > 0;
    if (have_m) {
        // learned sketches of the rows that go through the cache: rows first .. n_prompt - 1 of every unit
        const void *krows = K;
        if constexpr (std::is_same_v<T, bf16_t>) {
            if (first > 0) {
                const size_t pieces = (size_t)pb.units * tail * pb.d / 8;
                hipLaunchKernelGGL(dec_gather_rows_kernel, dim3((unsigned)((pieces + kThreads - 1) / kThreads)),
                                   dim3(kThreads), 0, s, (const bf16_t *)K, (bf16_t *)ktail, pb.d, n_prompt, first, tail,
                                   pieces);
                PSF_LAUNCH_CHECK();
                krows = ktail;
            }
        }
        Problem part = pb;
        part.n = tail;
        st = general_sketch_f32(part, krows, G, m_tail, s);
        if (st != PSF_OK) return st;
    }
    const DecSketchArgs ska{G, pb.g_len, pb.heads, pb.per_head ? 1 : 0, pb.r};
    for (int pos0 = first; pos0 < n_prompt; pos0 += pb.b) {
        const int count = n_prompt - pos0 < pb.b ? n_prompt - pos0 : pb.b;
        const dim3 grid((unsigned)((count + kPrefillTokens - 1) / kPrefillTokens), (unsigned)pb.units);
        if (have_m)
            hipLaunchKernelGGL((dec_prefill_kernel<T, true>), grid, dim3(kThreads), 0, s, (const T *)K, (const T *)V,
                               (const float *)m_tail, state, L, pb.d, pb.dv, pb.p, pb.mcols, n_prompt, pos0, count,
                               first, tail, ska);
        else
            hipLaunchKernelGGL((dec_prefill_kernel<T, false>), grid, dim3(kThreads), 0, s, (const T *)K, (const T *)V,
                               (const float *)nullptr, state, L, pb.d, pb.dv, pb.p, pb.mcols, n_prompt, pos0, count,
                               first, tail, ska);
        PSF_LAUNCH_CHECK();
        if (count == pb.b) {
            st = launch_fold<T>(pb, L, state, s);
            if (st != PSF_OK) return st;
        }
    }
    return PSF_OK;
}

psf_status decode_prefill(const Problem &pb, const void *K, const void *V, const void *G, int n_prompt, void *state,
                          void *ws, hipStream_t s)
{
    return pb.bf16 ? prefill_launch<bf16_t>(pb, K, V, G, n_prompt, (float *)state, ws, s)
                   : prefill_launch<float>(pb, K, V, G, n_prompt, (float *)state, ws, s);
}

psf_status decode_step(const Problem &pb, const void *q, const void *k, const void *v, const void *G, int pos,
                       void *state, void *o, hipStream_t s)
{
    return pb.bf16 ? step_launch<bf16_t>(pb, q, k, v, G, pos, (float *)state, o, s)
                   : step_launch<float>(pb, q, k, v, G, pos, (float *)state, o, s);
}

}  // namespace psf
