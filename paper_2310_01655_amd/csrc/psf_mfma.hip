// bf16 MFMA path of libpsf for gfx950 (MI355X): causal polynomial-sketch attention with the
// block lower-triangular algorithm of PolySketchFormer (arXiv 2310.01655, Sections 3.1, 3.2).
//
// Kernels (R = sketch size r, D = head size d = dv, b = block size, t = n/b):
//   k_prep         degree 4 with Gaussian sketches: Algorithm 1 on bf16 MFMA for the query rows
//                  (m(Q) row-major bf16), for the key rows (m(K) as "token octets", see below, and
//                  the partial sums S = m(K)^T m(K) per workgroup: the "ones" column of
//                  H_l = phi'(K_l)^T [V_l | 1], because phi' = m (x) m) and V -> [n/8][D][8] bf16,
//                  as roles of two launches (queries + values at four workgroups per CU, keys
//                  at two); the sketch matrices are transposed on their way into LDS.  m(K) is
//                  stored as fp32 octets [n/8][2][R][4], or, for the half-precision state
//                  kernel, as fp16 octets [n/8][R][8] scaled by a power of two per 128 tokens.
//   k_transpose_g, k_sketch, k_v_octets
//                  the same steps as separate launches: degree 8 (two levels, the first level's
//                  accumulators are the second level's operands) and the backward pass.
//   k_den_scan     prefix of the S partials over blocks, stored as bf16 hi + lo MFMA operands.
//   k_state        running prefix state Z = sum phi'(k_j) v_j^T kept in MFMA accumulators while
//                  one workgroup walks the blocks in order; phi'(k_j) = m_j (x) m_j is expanded
//                  in registers (one operand broadcast across lanes with DPP) and never
//                  written to memory.  A bf16 snapshot Z_{l+1} is stored after each block, so
//                  the exclusive scan over blocks (Section 3.1) costs nothing extra.  Z is
//                  symmetric in its two sketch indices; for d = 64 only the half the output
//                  kernel reads is computed.  k_state_two_waves: the same with two waves per
//                  SIMD that split the token steps, for calls with a single block per unit.
//   k_out          per 256-token tile: exact in-block weights lt((Q_l K_l^T)^p) [V_l | 1]
//                  (Section 3.2) kept in registers, plus phi'(Q_l) Z_l with phi'(q_i) expanded
//                  in registers as the MFMA operand, then the division by 1 + denominator
//                  (Section 3).  NONCAUSAL instantiation (Section 2.2): no in-block phase, one
//                  state for all tokens.  PART = 1 / 2: the in-block part alone (fp32 rows and
//                  row sums left in the workspace) and the cross-block part that finishes them.
//   k_state_and_in_block
//                  d = r = 64, exact in-block weights, at most one state workgroup per CU: one
//                  launch whose workgroups take one of four roles by index -- the state kernel
//                  (in half precision when k_prep left fp16 sketches: state_f16_workgroup),
//                  the denominator scan, the in-block part of the output (k_out's PART 1) and
//                  the query sketch -- so that the in-block tiles fill the SIMD slots the
//                  state workgroups (one wave per SIMD) leave empty; k_out PART 2 follows.
//   k_learned_prep, k_learned_sketch
//                  Algorithm 2 (learned sketches) of degree 4 and 8 with d = 64 or 128 on MFMA; other learned
//                  cases take m(x) from the general fp32 kernel through k_m_to_bf16 /
//                  k_m_to_octets_and_partials.
//   psf_mfma_bwd.inl (included below): the backward pass for d = 64, p = 4.
//
// MFMA v_mfma_f32_32x32x16_bf16 operand layout used throughout (lane = 32*h + x, x < 32):
//   A[i][k]: lane x = i, half h supplies k = 8h..8h+7 (8 bf16 per lane)
//   B[k][j]: lane x = j, half h supplies k = 8h..8h+7
//   D[i][j]: lane x = j, register v holds row i = 8*(v/4) + 4*h + (v%4)
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "psf_internal.h"

namespace psf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWg = 256;          // 4 wavefronts
constexpr int kStateRing = 4;     // staged chunks per workgroup in k_state (ring of LDS buffers)

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 cvt8(f32x8 v) { return __builtin_convertvector(v, bf16x8); }
__device__ __forceinline__ bf16x4 cvt4(f32x4 v) { return __builtin_convertvector(v, bf16x4); }

__device__ __forceinline__ bf16x8 cvt8_from16(const f32x16 &v, int first)
{
    f32x8 t;
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = v[first + e];
    return cvt8(t);
}

template <int... Js, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Js...>, F &&f)
{
    (f(std::integral_constant<int, Js>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

template <int LANE>
__device__ __forceinline__ float row_bcast(float v)
{
    // value of lane LANE of each row of 16 lanes, delivered to all lanes of that row
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v),
                                                                  0x150 + LANE, 0xf, 0xf, false));
}

__device__ __forceinline__ float pow_p(float x, int p)
{
    x *= x;                 // p is 2, 4 or 8 here
    if (p >= 4) x *= x;
    if (p == 8) x *= x;
    return x;
}

// Direct global -> LDS copy of 16 bytes per lane: lane i of the wave lands at lds_wave_base +
// 16*i.  Completion is tracked by vmcnt; callers wait before the barrier that publishes it.
__device__ __forceinline__ void dma16(const void *gsrc_lane, void *lds_wave_base)
{
    // Written as assembly so that the compiler does not tie later LDS reads to these copies
    // with a full vmcnt(0) wait; callers count the copies in flight themselves (wait_vmem_le).
    // m0 carries the LDS destination; nothing else in these kernels uses m0.
    const uint32_t lds_off = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds_wave_base;
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gsrc_lane), "s"(__builtin_amdgcn_readfirstlane(lds_off))
                 : "memory");
}
// Same copy with the address split into a wave-uniform base (scalar registers) and a 32-bit
// per-lane byte offset: a loop that walks the base then spends no vector instructions on it.
// The destination is given as an LDS byte address (see lds_address).
__device__ __forceinline__ void dma16_sbase(const void *gsrc_uniform, uint32_t lane_byte_off, uint32_t lds_wave_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_byte_off), "s"(gsrc_uniform), "s"(__builtin_amdgcn_readfirstlane(lds_wave_addr))
                 : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
__device__ __forceinline__ void wait_all_memory() { __builtin_amdgcn_s_waitcnt(0); }
// Wait until at most N vector-memory operations of this wave are outstanding (they complete in
// order, so everything older has landed); LDS/scalar counters are left alone.
template <int N>
__device__ __forceinline__ void wait_vmem_le()
{
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14));
}

// ------------------------------------------------------------------------------------
// Sketch matrices transposed once: Gt[set][mat][c][e] = G[set][mat][e][c], so that the sketch
// kernel stages MFMA operands (8 consecutive e per lane) with 16-byte copies.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWg) void k_transpose_g(const bf16_t *__restrict__ G,
                                                     bf16_t *__restrict__ Gt, int d, int r, int p,
                                                     size_t g_len)
{
    const int mat = blockIdx.x, set = blockIdx.y;
    const int n_first = p / 2;
    const int rows = mat < n_first ? d : r;
    const size_t off = mat < n_first ? (size_t)mat * d * r
                                     : (size_t)n_first * d * r + (size_t)(mat - n_first) * r * r;
    const bf16_t *g = G + set * g_len + off;
    bf16_t *gt = Gt + set * g_len + off;
    for (int idx = threadIdx.x; idx < rows * r; idx += kWg) {
        const int c = idx / rows, e = idx % rows;
        gt[idx] = g[(size_t)e * r + c];
    }
}

// ------------------------------------------------------------------------------------
// Algorithm 1 on MFMA.  One wave sketches 32 tokens at a time; a workgroup walks
// `tiles_per_wg` consecutive 128-token tiles of one unit so that the sketch matrices staged
// in LDS are reused.
//   QSIDE: results in D^T orientation (lane = token): writes M_rm [rows][R] bf16.
//   !QSIDE: results in D orientation (lane = sketch column): writes M8 [U][n/8][2][R][4] fp32
//          (token octet, half of the octet, sketch column, 4 tokens: conflict-free LDS reads)
//          and the workgroup's partial S = sum_j m_j m_j^T (the "ones" column of the block
//          states, since phi' = m (x) m) to Spart [U][n / tokens_per_wg][R][R].
// ------------------------------------------------------------------------------------
template <int D, int R>
struct SketchLds {
    static constexpr int kPitch = (D > R ? D : R) + 8;     // bf16 elements per transposed row
    bf16_t gt[2][R * kPitch];
};

template <int D, int R, int ROWS>
__device__ __forceinline__ void stage_gt(bf16_t *dst, const bf16_t *gt)
{
    // gt is [R][ROWS] (already transposed); rows are padded to kPitch in LDS
    constexpr int PITCH = SketchLds<D, R>::kPitch;
    constexpr int VEC = ROWS / 8;
    for (int idx = threadIdx.x; idx < R * VEC; idx += kWg) {
        const int c = idx / VEC, part = idx % VEC;
        *(uint4 *)&dst[c * PITCH + 8 * part] = *(const uint4 *)&gt[(size_t)c * ROWS + 8 * part];
    }
}

// acc[ct] = G^T X^T restricted to 32 tokens; xfr are the operand fragments of X.
template <int D, int R, int KSTEPS, bool TOKEN_LANES>
__device__ __forceinline__ void project(const bf16_t *gt, const bf16x8 *xfr, f32x16 *acc, int x,
                                        int h)
{
    constexpr int PITCH = SketchLds<D, R>::kPitch;
#pragma unroll
    for (int ct = 0; ct < R / 32; ++ct) {
        f32x16 c = {0};
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const bf16x8 g = *(const bf16x8 *)&gt[(32 * ct + x) * PITCH + 16 * s + 8 * h];
            c = TOKEN_LANES ? mfma32(g, xfr[s], c) : mfma32(xfr[s], g, c);
        }
        acc[ct] = c;
    }
}

// Second-level projection: operand fragments of M (from accumulators, k index permuted as
// 16s + 8*(e/4) + 4h + e%4) against G (R x R), same permutation on the G side.
template <int D, int R, bool TOKEN_LANES>
__device__ __forceinline__ void project_inner(const bf16_t *gt, const bf16x8 *mfr, f32x16 *acc,
                                              int x, int h)
{
    constexpr int PITCH = SketchLds<D, R>::kPitch;
#pragma unroll
    for (int ct = 0; ct < R / 32; ++ct) {
        f32x16 c = {0};
#pragma unroll
        for (int s = 0; s < R / 16; ++s) {
            const bf16x4 lo = *(const bf16x4 *)&gt[(32 * ct + x) * PITCH + 16 * s + 4 * h];
            const bf16x4 hi = *(const bf16x4 *)&gt[(32 * ct + x) * PITCH + 16 * s + 8 + 4 * h];
            bf16x8 g;
#pragma unroll
            for (int e = 0; e < 4; ++e) { g[e] = lo[e]; g[4 + e] = hi[e]; }
            c = TOKEN_LANES ? mfma32(g, mfr[s], c) : mfma32(mfr[s], g, c);
        }
        acc[ct] = c;
    }
}

template <int D, int R, int P, bool QSIDE>
__global__ __launch_bounds__(kWg) void k_sketch(const bf16_t *__restrict__ X,
                                                const bf16_t *__restrict__ Gt, int n, int heads,
                                                int per_head, size_t g_len, int tiles_per_wg,
                                                bf16_t *__restrict__ M_rm, float *__restrict__ M8,
                                                float *__restrict__ Spart)
{
    __shared__ __attribute__((aligned(16))) SketchLds<D, R> lds;
    __shared__ float red[QSIDE ? 1 : 4][QSIDE ? 1 : 32][33];
    __shared__ __attribute__((aligned(16))) bf16_t qtile[QSIDE ? 4 : 1][QSIDE ? 32 : 1][R + 8];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int x = lane & 31, h = lane >> 5;
    const size_t tok_wg0 = (size_t)blockIdx.x * tiles_per_wg * 128;   // global token (row) index
    const int u = (int)(tok_wg0 / n);
    const bf16_t *g = Gt + (per_head ? (size_t)(u % heads) * g_len : 0);
    const float scale = sqrtf(1.0f / (float)R);
    constexpr int KS = D / 16, NT = R / 32;

    f32x16 sacc[QSIDE ? 1 : NT][QSIDE ? 1 : NT];
    if (!QSIDE) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) sacc[i][j] = f32x16{0};
    }

#pragma unroll 1
    for (int tile = 0; tile < tiles_per_wg; ++tile) {
        const size_t row0 = tok_wg0 + (size_t)tile * 128 + wave * 32;   // this wave's 32 tokens
        bf16x8 xfr[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s)
            xfr[s] = *(const bf16x8 *)&X[(row0 + x) * D + 16 * s + 8 * h];

        f32x16 m[NT];
        if (P == 4) {
            if (tile == 0) {
                stage_gt<D, R, D>(lds.gt[0], g);
                stage_gt<D, R, D>(lds.gt[1], g + (size_t)D * R);
                __syncthreads();
            }
            f32x16 a0[NT], a1[NT];
            project<D, R, KS, QSIDE>(lds.gt[0], xfr, a0, x, h);
            project<D, R, KS, QSIDE>(lds.gt[1], xfr, a1, x, h);
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) m[ct] = scale * (a0[ct] * a1[ct]);
        } else {
            // degree 4 = p/2: two independent degree-2 sketches, then one more level
            bf16x8 m1fr[R / 16], m2fr[R / 16];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                __syncthreads();
                stage_gt<D, R, D>(lds.gt[0], g + (size_t)(2 * half) * D * R);
                stage_gt<D, R, D>(lds.gt[1], g + (size_t)(2 * half + 1) * D * R);
                __syncthreads();
                f32x16 a0[NT], a1[NT];
                project<D, R, KS, true>(lds.gt[0], xfr, a0, x, h);
                project<D, R, KS, true>(lds.gt[1], xfr, a1, x, h);
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) {
                    const f32x16 mm = scale * (a0[ct] * a1[ct]);
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        if (half == 0) m1fr[2 * ct + q] = cvt8_from16(mm, 8 * q);
                        else m2fr[2 * ct + q] = cvt8_from16(mm, 8 * q);
                    }
                }
            }
            __syncthreads();
            const bf16_t *gi = g + (size_t)4 * D * R;
            stage_gt<D, R, R>(lds.gt[0], gi);
            stage_gt<D, R, R>(lds.gt[1], gi + (size_t)R * R);
            __syncthreads();
            f32x16 a0[NT], a1[NT];
            project_inner<D, R, QSIDE>(lds.gt[0], m1fr, a0, x, h);
            project_inner<D, R, QSIDE>(lds.gt[1], m2fr, a1, x, h);
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) m[ct] = scale * (a0[ct] * a1[ct]);
        }

        if (QSIDE) {
            // lane = token x, register v = sketch column 32ct + 8(v/4) + 4h + v%4.  The 32 x R
            // tile goes through LDS so that the row-major store is contiguous (16 bytes per lane).
            bf16_t *tile = qtile[wave][0];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int c0 = 32 * ct + 8 * gq + 4 * h;
                    f32x4 q4 = {m[ct][4 * gq], m[ct][4 * gq + 1], m[ct][4 * gq + 2], m[ct][4 * gq + 3]};
                    *(bf16x4 *)&tile[x * (R + 8) + c0] = cvt4(q4);
                }
            __builtin_amdgcn_s_waitcnt((0x3F & 0xF) | (0x7 << 4) | (0x0 << 8) | ((0x3F >> 4) << 14));   // own LDS writes
#pragma unroll
            for (int i = 0; i < 32 * R / 8 / 64; ++i) {
                const int w = i * 64 + lane, tok = w / (R / 8), part = w % (R / 8);
                *(uint4 *)&M_rm[(row0 + tok) * R + 8 * part] = *(const uint4 *)&tile[tok * (R + 8) + 8 * part];
            }
        } else {
            // lane = sketch column 32ct + x, register v = token 8(v/4) + 4h + v%4
#pragma unroll
            for (int ct = 0; ct < NT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int c = 32 * ct + x;
                    f32x4 q4 = {m[ct][4 * gq], m[ct][4 * gq + 1], m[ct][4 * gq + 2], m[ct][4 * gq + 3]};
                    const size_t oct = (row0 >> 3) + gq;
                    *(f32x4 *)&M8[((oct * 2 + h) * R + c) * 4] = q4;
                    if (M_rm)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            M_rm[(row0 + 8 * gq + 4 * h + j) * R + c] = f32_to_bf16(q4[j]);
                }
            // S += M^T M over these 32 tokens: the accumulator registers, taken 8 at a time, are
            // valid A and B fragments at once (k = token, same permutation on both sides)
#pragma unroll
            for (int sp = 0; sp < 2; ++sp) {
                bf16x8 f[NT];
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) f[ct] = cvt8_from16(m[ct], 8 * sp);
#pragma unroll
                for (int i = 0; i < NT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j) sacc[i][j] = mfma32(f[i], f[j], sacc[i][j]);
            }
        }
    }

    if (!QSIDE) {
        float *out = Spart + (size_t)blockIdx.x * R * R;
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                __syncthreads();
#pragma unroll
                for (int v = 0; v < 16; ++v) red[wave][8 * (v / 4) + 4 * h + (v % 4)][x] = sacc[i][j][v];
                __syncthreads();
                for (int idx = threadIdx.x; idx < 32 * 32; idx += kWg) {
                    const int a = idx / 32, c = idx % 32;
                    out[(size_t)(32 * i + a) * R + 32 * j + c] =
                        red[0][a][c] + red[1][a][c] + red[2][a][c] + red[3][a][c];
                }
            }
    }
}

// V [rows][D] -> V8 [rows/8][D][8] (bf16 bits moved, not converted)
template <int D>
__global__ __launch_bounds__(kWg) void k_v_octets(const bf16_t *__restrict__ V,
                                                  bf16_t *__restrict__ V8, size_t octets)
{
    const size_t idx = (size_t)blockIdx.x * kWg + threadIdx.x;
    if (idx >= octets * D) return;
    const size_t oct = idx / D;
    const int c = (int)(idx % D);
    uint16_t tmp[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) tmp[j] = V[(oct * 8 + j) * D + c];
    uint4 pk;
    pk.x = tmp[0] | ((uint32_t)tmp[1] << 16);
    pk.y = tmp[2] | ((uint32_t)tmp[3] << 16);
    pk.z = tmp[4] | ((uint32_t)tmp[5] << 16);
    pk.w = tmp[6] | ((uint32_t)tmp[7] << 16);
    *(uint4 *)&V8[idx * 8] = pk;
}

// ------------------------------------------------------------------------------------
// Everything the state and output kernels need (degree 4, Gaussian sketches).  A workgroup
// takes one role on one part of the rows (a part = 128 * tiles_per_wg tokens of one unit):
// 0 = sketch of the query rows (m(Q) as bf16 rows), 1 = sketch of the key rows (m(K) as fp32
// token octets + the part's S = m^T m), 2 = the value rows as token octets.  The sketch
// matrices are read as given, [d][r] row-major, and transposed on their way into LDS (once per
// workgroup), so no transposed copy is needed.
// ------------------------------------------------------------------------------------
template <int D, int R>
struct PrepLds {
    SketchLds<D, R> g;
    union {
        float red[4][32][33];                        // key role: S partial reduction
        bf16_t qtile[4][32][R + 8];                  // row-major store staging (query role; bf16 rows of m(K))
    } u;
    float tmax[8];                                   // fp16 key role: the four waves' maxima, two tiles in flight
};

template <int D, int R>
__device__ __forceinline__ void stage_g_transposing(bf16_t *dst, const bf16_t *g)
{
    // g is [D][R] row-major; dst[c * PITCH + e] = g[e][c]
    constexpr int PITCH = SketchLds<D, R>::kPitch;
    constexpr int VEC = R / 8;
    for (int idx = threadIdx.x; idx < D * VEC; idx += kWg) {
        const int e = idx / VEC, part = idx % VEC;
        const uint4 raw = *(const uint4 *)&g[(size_t)e * R + 8 * part];
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 8; ++i)
            dst[(8 * part + i) * PITCH + e] = (bf16_t)(w[i / 2] >> (16 * (i % 2)));
    }
}

template <int D, int R, bool QSIDE>
__device__ __forceinline__ void prep_sketch_role(PrepLds<D, R> &lds, const bf16_t *__restrict__ X,
                                                 const bf16_t *__restrict__ g, size_t tok_wg0, int tiles_per_wg,
                                                 bf16_t *__restrict__ M_rm, float *__restrict__ M8,
                                                 float *__restrict__ Spart_out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int x = lane & 31, h = lane >> 5;
    const float scale = sqrtf(1.0f / (float)R);
    constexpr int KS = D / 16, NT = R / 32;

    f32x16 sacc[QSIDE ? 1 : NT][QSIDE ? 1 : NT];
    if (!QSIDE) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) sacc[i][j] = f32x16{0};
    }
    // first tile's operands are on their way while the matrices are staged
    bf16x8 xfr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) xfr[s] = *(const bf16x8 *)&X[(tok_wg0 + wave * 32 + x) * D + 16 * s + 8 * h];
    stage_g_transposing<D, R>(lds.g.gt[0], g);
    stage_g_transposing<D, R>(lds.g.gt[1], g + (size_t)D * R);
    __syncthreads();

#pragma unroll 1
    for (int tile = 0; tile < tiles_per_wg; ++tile) {
        const size_t row0 = tok_wg0 + (size_t)tile * 128 + wave * 32;   // this wave's 32 tokens
        f32x16 a0[NT], a1[NT], m[NT];
        project<D, R, KS, QSIDE>(lds.g.gt[0], xfr, a0, x, h);
        project<D, R, KS, QSIDE>(lds.g.gt[1], xfr, a1, x, h);
        // Operands of the next tile (the last tile loads its own rows again: no branch here).
        // A conditional block between the MFMAs above and the first read of their results
        // made the compiler count the wait states of the skipped loads: on the path that skips
        // them the last accumulator registers were read before the matrix pipe had written
        // them.  Straight-line code gets the full wait.
        {
            const size_t nrow = row0 + (tile + 1 < tiles_per_wg ? 128 : 0);
#pragma unroll
            for (int s = 0; s < KS; ++s) xfr[s] = *(const bf16x8 *)&X[(nrow + x) * D + 16 * s + 8 * h];
        }
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) m[ct] = scale * (a0[ct] * a1[ct]);

        if (QSIDE) {
            // lane = token x, register v = sketch column 32ct + 8(v/4) + 4h + v%4; through LDS so
            // that the row-major store is 16 contiguous bytes per lane
            bf16_t *qt = lds.u.qtile[wave][0];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int c0 = 32 * ct + 8 * gq + 4 * h;
                    f32x4 q4 = {m[ct][4 * gq], m[ct][4 * gq + 1], m[ct][4 * gq + 2], m[ct][4 * gq + 3]};
                    *(bf16x4 *)&qt[x * (R + 8) + c0] = cvt4(q4);
                }
            __builtin_amdgcn_s_waitcnt((0x3F & 0xF) | (0x7 << 4) | (0x0 << 8) | ((0x3F >> 4) << 14));   // own LDS writes
#pragma unroll
            for (int i = 0; i < 32 * R / 8 / 64; ++i) {
                const int w = i * 64 + lane, tok = w / (R / 8), part = w % (R / 8);
                *(uint4 *)&M_rm[(row0 + tok) * R + 8 * part] = *(const uint4 *)&qt[tok * (R + 8) + 8 * part];
            }
        } else {
            // lane = sketch column 32ct + x, register v = token 8(v/4) + 4h + v%4
#pragma unroll
            for (int ct = 0; ct < NT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int c = 32 * ct + x;
                    f32x4 q4 = {m[ct][4 * gq], m[ct][4 * gq + 1], m[ct][4 * gq + 2], m[ct][4 * gq + 3]};
                    const size_t oct = (row0 >> 3) + gq;
                    *(f32x4 *)&M8[((oct * 2 + h) * R + c) * 4] = q4;
                    if (M_rm)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            M_rm[(row0 + 8 * gq + 4 * h + j) * R + c] = f32_to_bf16(q4[j]);
                }
#pragma unroll
            for (int sp = 0; sp < 2; ++sp) {              // S += M^T M over these 32 tokens
                bf16x8 f[NT];
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) f[ct] = cvt8_from16(m[ct], 8 * sp);
#pragma unroll
                for (int i = 0; i < NT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j) sacc[i][j] = mfma32(f[i], f[j], sacc[i][j]);
            }
        }
    }

    if (!QSIDE) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                __syncthreads();
#pragma unroll
                for (int v = 0; v < 16; ++v) lds.u.red[wave][8 * (v / 4) + 4 * h + (v % 4)][x] = sacc[i][j][v];
                __syncthreads();
                for (int idx = threadIdx.x; idx < 32 * 32; idx += kWg) {
                    const int a = idx / 32, c = idx % 32;
                    Spart_out[(size_t)(32 * i + a) * R + 32 * j + c] =
                        lds.u.red[0][a][c] + lds.u.red[1][a][c] + lds.u.red[2][a][c] + lds.u.red[3][a][c];
                }
            }
    }
}

// Key rows for the half-precision state kernel: m(K) as fp16 token octets [rows/8][R][8],
// multiplied by a power of two alpha chosen per 128-token tile so that every |alpha m| < 1
// (alpha itself goes to scale_out, one float per tile; powers of two keep the scaling exact and
// the state kernel divides it out again), and the part's S = m^T m from the unscaled values.
// fp16 carries more mantissa than the bf16 the products are rounded to elsewhere, but only 5
// exponent bits: the scale is what keeps rows of any norm inside them.
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// ROWS: also leave the unscaled sketch as bf16 rows in M_rm (a separate instantiation: the code
// for it costs the plain one a third workgroup per CU in registers).
template <int D, int R, bool ROWS>
__device__ __forceinline__ void prep_keys_f16_role(PrepLds<D, R> &lds, const bf16_t *__restrict__ X,
                                                   const bf16_t *__restrict__ g, size_t tok_wg0, int tiles_per_wg,
                                                   _Float16 *__restrict__ MKh, float *__restrict__ scale_out,
                                                   float *__restrict__ Spart_out, bf16_t *__restrict__ M_rm)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int x = lane & 31, h = lane >> 5;
    const float scale = sqrtf(1.0f / (float)R);
    constexpr int KS = D / 16, NT = R / 32;
    stage_g_transposing<D, R>(lds.g.gt[0], g);
    stage_g_transposing<D, R>(lds.g.gt[1], g + (size_t)D * R);
    __syncthreads();

    auto sketch_tile = [&](int tile, f32x16 *m) {
        const size_t row0 = tok_wg0 + (size_t)tile * 128 + wave * 32;
        bf16x8 xfr[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) xfr[s] = *(const bf16x8 *)&X[(row0 + x) * D + 16 * s + 8 * h];
        f32x16 a0[NT], a1[NT];
        project<D, R, KS, false>(lds.g.gt[0], xfr, a0, x, h);
        project<D, R, KS, false>(lds.g.gt[1], xfr, a1, x, h);
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) m[ct] = scale * (a0[ct] * a1[ct]);
    };

    f32x16 sacc[NT][NT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) sacc[i][j] = f32x16{0};
    float *tile_max = lds.tmax;                            // [2][4]
#pragma unroll 1
    for (int tile = 0; tile < tiles_per_wg; ++tile) {
        const size_t row0 = tok_wg0 + (size_t)tile * 128 + wave * 32;
        f32x16 m[NT];
        sketch_tile(tile, m);
        float mx = 0.f;
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, fabsf(m[ct][v]));
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        if (lane == 0) tile_max[(tile & 1) * 4 + wave] = mx;
        __syncthreads();                                   // (the slot is written again two tiles later: one barrier per tile)
        const float *tm = tile_max + (tile & 1) * 4;
        mx = fmaxf(fmaxf(tm[0], tm[1]), fmaxf(tm[2], tm[3]));
        // mx = f 2^e with f in [0.5, 1)  ->  alpha = 2^-e (1 for a tile of zeros).  The exponent of
        // alpha is kept within +-40, so that its square and the ratio of two squares stay finite
        // in fp32; rows beyond 2^40 times the unit scale are not a case to serve.
        const int ebits = min(max((int)((__float_as_uint(mx) >> 23) & 0xffu), 126 - 40), 126 + 40);
        const float alpha = mx > 0.f ? __uint_as_float((uint32_t)(253 - ebits) << 23) : 1.0f;
        if (threadIdx.x == 0) scale_out[tile] = alpha;
        // lane = sketch column 32ct + x, register v = token 8(v/4) + 4h + v%4: half an octet per
        // register quad, 8 bytes per lane
#pragma unroll
        for (int ct = 0; ct < NT; ++ct)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int c = 32 * ct + x;
                const size_t oct = (row0 >> 3) + gq;
                f16x4 q4 = {(_Float16)(alpha * m[ct][4 * gq]), (_Float16)(alpha * m[ct][4 * gq + 1]),
                            (_Float16)(alpha * m[ct][4 * gq + 2]), (_Float16)(alpha * m[ct][4 * gq + 3])};
                *(f16x4 *)&MKh[(oct * R + c) * 8 + 4 * h] = q4;
            }
        if constexpr (ROWS) {
            // unscaled bf16 rows as well (the backward pass reads them): through LDS, so that the
            // row-major store is 16 contiguous bytes per lane
            bf16_t *qt = lds.u.qtile[wave][0];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    qt[(8 * (v / 4) + 4 * h + v % 4) * (R + 8) + 32 * ct + x] = f32_to_bf16(m[ct][v]);
            __builtin_amdgcn_s_waitcnt((0x3F & 0xF) | (0x7 << 4) | (0x0 << 8) | ((0x3F >> 4) << 14));   // own LDS writes
#pragma unroll
            for (int i = 0; i < 32 * R / 8 / 64; ++i) {
                const int w = i * 64 + lane, tok = w / (R / 8), part = w % (R / 8);
                *(uint4 *)&M_rm[(row0 + tok) * R + 8 * part] = *(const uint4 *)&qt[tok * (R + 8) + 8 * part];
            }
        }
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {              // S += M^T M over these 32 tokens
            bf16x8 f[NT];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) f[ct] = cvt8_from16(m[ct], 8 * sp);
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) sacc[i][j] = mfma32(f[i], f[j], sacc[i][j]);
        }
    }
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) lds.u.red[wave][8 * (v / 4) + 4 * h + (v % 4)][x] = sacc[i][j][v];
            __syncthreads();
            for (int idx = threadIdx.x; idx < 32 * 32; idx += kWg) {
                const int a = idx / 32, c = idx % 32;
                Spart_out[(size_t)(32 * i + a) * R + 32 * j + c] =
                    lds.u.red[0][a][c] + lds.u.red[1][a][c] + lds.u.red[2][a][c] + lds.u.red[3][a][c];
            }
        }
}

// KEYS = false: roles 0 and 2 alternate (few registers, four workgroups per CU); KEYS = true: role 1
// alone (its S accumulators make it the register-heavy one; as one launch with the others it
// would pull them down to its occupancy).
// F16: for the half-precision state kernel -- role 1 writes fp16 key sketches and their scale
// (prep_keys_f16_role; MK8 then points to them, Kscale gets one float per 128-token tile), role 2 also
// writes the value rows as fp16 token octets (V8h; magnitudes beyond the fp16 range saturate).
template <int D, int R, bool KEYS, bool F16 = false, bool ROWS = false>
__global__ __launch_bounds__(kWg, KEYS ? 2 : 4) void k_prep(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                              const bf16_t *__restrict__ V, const bf16_t *__restrict__ G,
                                              int n, int heads, int per_head, size_t g_len, int tiles_per_wg,
                                              bf16_t *__restrict__ MQ, float *__restrict__ MK8,
                                              bf16_t *__restrict__ MK_rm, float *__restrict__ Spart,
                                              bf16_t *__restrict__ V8, int with_q,
                                              float *__restrict__ Kscale, _Float16 *__restrict__ V8h)
{
    // (with_q == 0: the query rows are sketched elsewhere; every workgroup takes role 2)
    __shared__ __attribute__((aligned(16))) PrepLds<D, R> lds;
    const int role = KEYS ? 1 : (with_q ? 2 * (int)(blockIdx.x % 2) : 2);
    const size_t part = (KEYS || !with_q) ? blockIdx.x : blockIdx.x / 2;
    const size_t tok_wg0 = part * (size_t)tiles_per_wg * 128;           // first row of the part (all units)
    if (!KEYS && role == 2) {
        // value rows -> token octets [rows/8][D][8]: one 16-byte store per thread and step
        // (UN outputs per thread and step, all their loads issued before the first is used: the
        // role is bound by memory latency otherwise)
        constexpr int UN = 4;
        const size_t first = tok_wg0 / 8 * D, count = (size_t)tiles_per_wg * 16 * D;   // count % (UN * kWg) == 0
        static_assert((16 * D) % (UN * kWg) == 0, "whole steps per 128-token tile");
        for (size_t i0 = threadIdx.x; i0 < count; i0 += UN * kWg) {
            uint16_t tmp[UN][8];
#pragma unroll
            for (int q = 0; q < UN; ++q) {
                const size_t idx = first + i0 + (size_t)q * kWg, oct = idx / D;
                const int c = (int)(idx % D);
#pragma unroll
                for (int j = 0; j < 8; ++j) tmp[q][j] = V[(oct * 8 + j) * D + c];
            }
#pragma unroll
            for (int q = 0; q < UN; ++q) {
                const size_t idx = first + i0 + (size_t)q * kWg;
                uint4 pk;
                pk.x = tmp[q][0] | ((uint32_t)tmp[q][1] << 16);
                pk.y = tmp[q][2] | ((uint32_t)tmp[q][3] << 16);
                pk.z = tmp[q][4] | ((uint32_t)tmp[q][5] << 16);
                pk.w = tmp[q][6] | ((uint32_t)tmp[q][7] << 16);
                *(uint4 *)&V8[idx * 8] = pk;
                if constexpr (F16) {
                    f16x8 hv;
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        hv[j] = (_Float16)fminf(fmaxf(bf16_to_f32(tmp[q][j]), -65504.f), 65504.f);
                    *(f16x8 *)&V8h[idx * 8] = hv;
                }
            }
        }
        return;
    }
    const int u = (int)(tok_wg0 / n);
    const bf16_t *g = G + (per_head ? (size_t)(u % heads) * g_len : 0);
    if constexpr (!KEYS)
        prep_sketch_role<D, R, true>(lds, Q, g, tok_wg0, tiles_per_wg, MQ, nullptr, nullptr);
    else if constexpr (F16)
        prep_keys_f16_role<D, R, ROWS>(lds, K, g, tok_wg0, tiles_per_wg, (_Float16 *)MK8, Kscale + part * tiles_per_wg,
                                       Spart + part * R * R, MK_rm);
    else
        prep_sketch_role<D, R, false>(lds, K, g, tok_wg0, tiles_per_wg, MK_rm, MK8, Spart + part * R * R);
}

// Prefix over the sketch kernel's per-workgroup partials of S, snapshotted at block boundaries
// and written as MFMA A-operands [R/8][R][8] bf16, split into hi + lo so that the denominator
// keeps ~16 mantissa bits.  Slot l holds sum over blocks 0..l, which is what block l+1 needs.
// (u, blk): unit and which 256 of its R * R entries this workgroup scans
template <int R>
__device__ __forceinline__ void den_scan_workgroup(const float *__restrict__ Spart, bf16_t *__restrict__ Shi,
                                                   bf16_t *__restrict__ Slo, int t, int parts_per_block,
                                                   int parts_per_unit, int u, int blk, bf16_t *xch)
{
    // One entry of S per thread, threads in the order of the partials (row-major [a][b']): a wave
    // reads 256 contiguous bytes of every partial.  At a block boundary the 256 results change
    // places through LDS (xch: 2 * kWg entries) so that they leave in the order of the output
    // layout [b'/8][a][8]: pieces of kWg / R rows x 8 columns, 16 bytes per row.
    static_assert(kWg % R == 0 && (R * R) % kWg == 0, "whole rows per workgroup");
    constexpr int ROWS = kWg / R;
    const int tid = threadIdx.x;
    const int e = blk * kWg + tid;
    const int a0 = blk * ROWS;
    const int within = tid % (ROWS * 8), oa = a0 + within / 8, obq = 8 * (tid / (ROWS * 8)) + within % 8;
    const int from = (oa - a0) * R + obq;                 // the thread that holds entry (oa, obq)
    const int dst = ((obq / 8) * R + oa) * 8 + obq % 8;
    const float *src = Spart + (size_t)u * parts_per_unit * R * R + e;
    const int total = (t - 1) * parts_per_block;
    float run = 0.f;
    constexpr int FLY = 8;                        // loads in flight per thread (32 measured slower)
    for (int w0 = 0; w0 < total; w0 += FLY) {
        float v[FLY];
#pragma unroll
        for (int i = 0; i < FLY; ++i) v[i] = (w0 + i < total) ? src[(size_t)(w0 + i) * R * R] : 0.f;
#pragma unroll
        for (int i = 0; i < FLY; ++i) {
            const int w = w0 + i;
            run += v[i];                          // zero past the end
            if (w < total && (w + 1) % parts_per_block == 0) {       // the same for every thread
                const int l = w / parts_per_block;
                const size_t base = ((size_t)u * (t - 1) + l) * R * R;
                const bf16_t hi = f32_to_bf16(run);
                xch[tid] = hi;
                xch[kWg + tid] = f32_to_bf16(run - bf16_to_f32(hi));
                __syncthreads();
                Shi[base + dst] = xch[from];
                Slo[base + dst] = xch[kWg + from];
                __syncthreads();
            }
        }
    }
}

template <int R>
__global__ __launch_bounds__(kWg) void k_den_scan(const float *__restrict__ Spart,
                                                  bf16_t *__restrict__ Shi, bf16_t *__restrict__ Slo,
                                                  int t, int parts_per_block, int parts_per_unit)
{
    __shared__ bf16_t xch[2 * kWg];
    den_scan_workgroup<R>(Spart, Shi, Slo, t, parts_per_block, parts_per_unit, blockIdx.y, blockIdx.x, xch);
}

// ------------------------------------------------------------------------------------
// Running prefix state.  Workgroup = (unit, group of AG = NA * 4 / NB sketch rows a); wave =
// (NA rows a) x (32 columns b') x (all D value columns).  Accumulator tile (a, ct):
// rows b' (A operand = phi'(k)^T generated in registers), columns c (B operand = V).
// ------------------------------------------------------------------------------------
template <int AI>
__device__ __forceinline__ bf16x8 gen_frag(const f32x4 &af, const f32x8 &bfv)
{
    // products m_j[a] * m_j[b'] for the 8 tokens of this lane's half; a is broadcast with DPP
    // from lane 8*(e/4) + AI of each row, which holds tokens 4*(e/4)..+3 of row a0 + AI.
    f32x8 p;
    p[0] = row_bcast<AI>(af[0]) * bfv[0];
    p[1] = row_bcast<AI>(af[1]) * bfv[1];
    p[2] = row_bcast<AI>(af[2]) * bfv[2];
    p[3] = row_bcast<AI>(af[3]) * bfv[3];
    p[4] = row_bcast<8 + AI>(af[0]) * bfv[4];
    p[5] = row_bcast<8 + AI>(af[1]) * bfv[5];
    p[6] = row_bcast<8 + AI>(af[2]) * bfv[6];
    p[7] = row_bcast<8 + AI>(af[3]) * bfv[7];
    return cvt8(p);
}

template <int CT>
struct StateOps {           // LDS operands of one 16-token step
    f32x4 af;               // m_j[a] source values (see gen_frag)
    f32x8 bfv;              // m_j[b'] for this lane's b' and 8 tokens
    bf16x8 vf[CT];          // V fragments (B operand)
};

// One 16-token step: for every tile of the wave, two things overlap -- the MFMAs that consume
// the fragment generated last, and the VALU work generating the next fragment (the first one
// of the following step comes from `nxt`).
template <int NA, int CT, int AI>
struct StateStep {
    static __device__ __forceinline__ void run(const StateOps<CT> &cur, const StateOps<CT> &nxt,
                                               bf16x8 &frag, f32x16 (*acc)[CT])
    {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[AI][ct] = mfma32(frag, cur.vf[ct], acc[AI][ct]);
        if constexpr (AI + 1 < NA) {
            frag = gen_frag<AI + 1>(cur.af, cur.bfv);
        } else {
            frag = gen_frag<0>(nxt.af, nxt.bfv);
        }
        // interleave: one MFMA, then half of the 12 VALU ops of the next fragment
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 12 / CT, 0);
        }
        if constexpr (AI + 1 < NA) StateStep<NA, CT, AI + 1>::run(cur, nxt, frag, acc);
    }
};

// LDS image of one staged chunk of the state kernel (TC tokens of m(k) and of v).  m sits there
// as planes of four tokens, [R][4] fp32 each, as in global memory.  The reads of m_j[a] for the
// DPP broadcast take the same few rows a from four planes at once; with R = 64 a plane is the
// 1 KB that one wave copies, and 64 bytes of padding per plane put those reads into different
// banks.
template <int R, int D, int TC>
struct StateLds {
    static constexpr int PLANE = R * 16;                          // four tokens of every sketch column
    static constexpr int PS = PLANE == 1024 ? PLANE + 64 : PLANE; // plane stride in LDS
    static constexpr int M_LDS = (TC / 4) * PS;
    static constexpr int BUF = (M_LDS + TC * D * 2 + 255) / 256 * 256;
    // LDS offset of the 1 KB that wave w copies of the 4 KB piece q of m
    static __device__ __forceinline__ uint32_t m_piece(int q, int w)
    {
        return PLANE == 1024 ? (uint32_t)((4 * q + w) * PS) : (uint32_t)(q * 4096 + w * 1024);
    }
};

// SYM: Z[a][b'] = Z[b'][a] and the output kernel reads, for sketch row a, only the 16-wide
// column ranges beta >= a / 16, so only those (a, beta) segments are computed: 16 (beta + 1)
// rows a per range beta, R/16 * (R/16 + 1) / 2 * 16 segments in all (160 of 256 for R = 64).
// A 32-row MFMA tile is two segments that share beta (lanes x < 16 and x >= 16 of the A operand
// carry different rows a), a wave owns NA = 2 tiles = four consecutive rows a of one beta, and
// the waves are numbered range by range: beta = 0 first (4 waves), then 1 (8 waves), ...
// NG = 2: eight waves, two per SIMD.  Waves w and w + 4 own the same tiles and take the even and
// the odd 16-token steps, so the vector instructions that generate one wave's next fragment
// run under the other wave's MFMAs; at a block boundary the two exchange partial sums through
// LDS so that each holds (and stores) the whole of one of the two tiles.
template <int R, int D, int NA, bool SYM, int TC, int NG>
__device__ __forceinline__ void state_body(const float *__restrict__ M8, const bf16_t *__restrict__ V8,
                                           bf16_t *__restrict__ Zg, int n, int b, int t, int u, int grp,
                                           unsigned char *lds_base)
{
    constexpr int NB = R / 32;                 // 32-wide b' ranges
    constexpr int AG = NA * 4 / NB;            // sketch rows a per workgroup (!SYM)
    constexpr int CT = D / 32;
    constexpr int NBUF = kStateRing;
    constexpr int STEPS = TC / 16 / NG;        // steps of one wave per chunk
    constexpr int PS = StateLds<R, D, TC>::PS;
    constexpr int M_BYTES = TC * R * 4, V_BYTES = TC * D * 2;
    constexpr int M_LDS = StateLds<R, D, TC>::M_LDS, BUF_BYTES = StateLds<R, D, TC>::BUF;
    constexpr int DMA_PER_CHUNK = (M_BYTES + V_BYTES) / 16 / (kWg * NG);
    constexpr int SEG = SYM ? 2 : 1;           // rows a per tile
    static_assert(M_BYTES % (4096 * NG) == 0 && V_BYTES % (4096 * NG) == 0, "whole 4 KB pieces per wave group");
    static_assert(NA <= 8, "DPP source lanes");
    static_assert(STEPS % 2 == 0, "operand ping-pong");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
    const int wave = wave8 & 3, wg2 = NG == 1 ? 0 : wave8 >> 2;  // tile owner; step parity (NG = 2)
    const int x = lane & 31, h = lane >> 5, n16 = lane & 15;
    // tiles of this wave: tile i holds the sketch rows a0 + i * SEG + (0..SEG-1); bcol is the
    // column b' of lane x
    int a0, beta = 0, bcol;
    if (SYM) {
        int w = grp * 4 + wave;                // wave of the unit
        while (w >= 4 * (beta + 1)) { w -= 4 * (beta + 1); ++beta; }
        a0 = w * NA * SEG;
        bcol = 16 * beta + (x & 15);
    } else {
        a0 = grp * AG + (wave / NB) * NA;
        beta = wave % NB;                      // 32-wide range here
        bcol = 32 * beta + x;
    }
    // lanes i and 8 + i of each row of 16 lanes fetch m_j[a] of tile i for the DPP broadcast;
    // with two segments per tile the odd rows (x >= 16) fetch the second row a
    const int a_src = a0 + min(n16 & 7, NA - 1) * SEG + (SYM ? (lane >> 4) & 1 : 0);
    const int q_src = n16 >> 3;

    f32x16 acc[NA][CT];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < CT; ++j) acc[i][j] = f32x16{0};

    const float *gm = M8 + (size_t)u * n * R;
    const bf16_t *gv = V8 + (size_t)u * n * D;
    const int chunks = (t - 1) * (b / TC), chunks_per_block = b / TC;

    // Ring slots are compile-time constants (the chunk loop dispatches on the slot), so every
    // LDS address below is a per-lane base plus an immediate and the copies take a scalar base.
    const uint32_t copy_off = (uint32_t)(tid & 255) * 16;     // lane's byte offset inside a 4 KB piece
    const uint32_t lds0 = lds_address(lds_base);
    auto stage = [&](auto slot_tag, int chunk) {              // straight copies: global layout == LDS layout
        constexpr int SLOT = decltype(slot_tag)::value;
        const unsigned char *sm = (const unsigned char *)(gm + (size_t)chunk * TC * R);
        const unsigned char *sv = (const unsigned char *)(gv + (size_t)chunk * TC * D);
        const uint32_t dst = lds0 + SLOT * BUF_BYTES;
        // (the wave groups share the pieces: group g copies pieces g, g + NG, ...)
#pragma unroll
        for (int qq = 0; qq < M_BYTES / 4096 / NG; ++qq) {
            const int q = qq * NG + wg2;
            dma16_sbase(sm + q * 4096, copy_off, dst + StateLds<R, D, TC>::m_piece(q, wave));
        }
#pragma unroll
        for (int qq = 0; qq < V_BYTES / 4096 / NG; ++qq) {
            const int q = qq * NG + wg2;
            dma16_sbase(sv + q * 4096, copy_off, dst + M_LDS + q * 4096 + wave * 1024);
        }
    };
    // step S of this wave is step NG * S + wg2 of the chunk: the parity sits in the lane bases
    const unsigned char *lane_b = lds_base + (h * 2 * PS + bcol * 16) + wg2 * 4 * PS;
    const unsigned char *lane_a = lds_base + ((h * 2 + q_src) * PS + a_src * 16) + wg2 * 4 * PS;
    const unsigned char *lane_v = lds_base + M_LDS + ((h * D + x) * 16) + wg2 * 2 * D * 16;
    auto load_ops = [&](auto slot_tag, auto step_tag) {
        constexpr int OFF = decltype(slot_tag)::value * BUF_BYTES;
        constexpr int S = decltype(step_tag)::value * NG;     // octet 2 (S + wg2) + h
        StateOps<CT> o;
        const f32x4 b_lo = *(const f32x4 *)(lane_b + OFF + S * 4 * PS);
        const f32x4 b_hi = *(const f32x4 *)(lane_b + OFF + S * 4 * PS + PS);
#pragma unroll
        for (int e = 0; e < 4; ++e) { o.bfv[e] = b_lo[e]; o.bfv[4 + e] = b_hi[e]; }
        o.af = *(const f32x4 *)(lane_a + OFF + S * 4 * PS);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) o.vf[ct] = *(const bf16x8 *)(lane_v + OFF + S * 2 * D * 16 + ct * 32 * 16);
        return o;
    };
    auto snapshot = [&](int l) {
        if constexpr (NG == 2) {
            // The two waves of a tile pair exchange partial sums through LDS, one value-column
            // tile per round: the wave of the even steps ends up with the whole of tile 0 and
            // keeps its running prefix, the other one with tile 1; each stores its tile below
            // and restarts the other tile from zero.  Buffer behind the ring:
            // [group][wave][register quad][lane] x 16 bytes.
            static_assert(NA == 2, "one tile per wave group");
            f32x4 *xb = (f32x4 *)(lds_base + NBUF * BUF_BYTES);
            f32x4 *mine = xb + ((wg2 * 4 + wave) * 4) * 64 + lane;
            const f32x4 *theirs = xb + (((wg2 ^ 1) * 4 + wave) * 4) * 64 + lane;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                // (the tile this wave gives away: index 1 - wg2)
                auto put = [&](const f32x16 &t) {
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4)
                        mine[v4 * 64] = f32x4{t[4 * v4], t[4 * v4 + 1], t[4 * v4 + 2], t[4 * v4 + 3]};
                };
                if (wg2) put(acc[0][ct]);
                else put(acc[1][ct]);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                auto take = [&](f32x16 &keep, f32x16 &given) {
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        const f32x4 q = theirs[v4 * 64];
#pragma unroll
                        for (int j = 0; j < 4; ++j) keep[4 * v4 + j] += q[j];
                    }
                    given = f32x16{0};
                };
                if (wg2) take(acc[1][ct], acc[0][ct]);
                else take(acc[0][ct], acc[1][ct]);
                if (ct + 1 < CT) {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
            }
        }
        // Z_{l+1} = sum over blocks 0..l, stored [a][b'/8][c][8] bf16.  Z[a][b'] = Z[b'][a]
        // (phi' = m (x) m), so the output kernel only contracts b' >= a: entries with b' > a are
        // stored doubled, b' < a as zero.
        bf16_t *z = Zg + ((size_t)u * (t - 1) + l) * R * R * D;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if (NG == 2 && i != wg2) continue;             // wave-uniform: the tile this wave holds in full
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    // accumulator rows 8 gq + 4 h + j: segment gq / 2 of the tile when SYM
                    const int a = a0 + i * SEG + (SYM ? gq / 2 : 0);
                    const int bq0 = SYM ? 16 * beta + 8 * (gq % 2) + 4 * h : 32 * beta + 8 * gq + 4 * h;
                    f32x4 q4;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float wsym = bq0 + j > a ? 2.f : (bq0 + j == a ? 1.f : 0.f);
                        q4[j] = acc[i][ct][4 * gq + j] * wsym;
                    }
                    *(bf16x4 *)&z[(((size_t)a * (R / 8) + bq0 / 8) * D + 32 * ct + x) * 8 + 4 * h] = cvt4(q4);
                }
        }
    };

    StateOps<CT> ops[2];
    ops[0] = load_ops(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    bf16x8 frag = gen_frag<0>(ops[0].af, ops[0].bfv);
    // One chunk = STEPS steps.  Operands of step s+1 are read from LDS at the start of step s.
    // Before the last step the next chunk must have landed for every wave (wait + barrier);
    // after that barrier nobody reads this chunk's buffer again, so the next iteration may
    // refill it.
    auto run_chunk = [&](auto slot_tag, int chunk) {
        constexpr int SLOT = decltype(slot_tag)::value;
        stage(std::integral_constant<int, (SLOT + NBUF - 1) % NBUF>{}, min(chunk + NBUF - 1, chunks - 1));
        static_for<STEPS>([&](auto s_tag) {
            constexpr int s = decltype(s_tag)::value;
            if (s == STEPS - 1) {
                // plain barrier: the copies are tracked by the explicit wait, and a fence
                // here would wait for the younger copies too
                wait_vmem_le<(NBUF - 2) * DMA_PER_CHUNK>();
                __builtin_amdgcn_s_barrier();
            }
            __builtin_amdgcn_sched_barrier(0);      // steps are scheduled one at a time
            if constexpr (s + 1 < STEPS)
                ops[(s + 1) & 1] = load_ops(slot_tag, std::integral_constant<int, s + 1>{});
            else
                ops[(s + 1) & 1] = load_ops(std::integral_constant<int, (SLOT + 1) % NBUF>{},
                                            std::integral_constant<int, 0>{});
            __builtin_amdgcn_sched_group_barrier(0x100, 3 + CT, 0);   // LDS reads first
            StateStep<NA, CT, 0>::run(ops[s & 1], ops[(s + 1) & 1], frag, acc);
        });
    };
    // The slots follow each other inside one loop body (a block holds a multiple of NBUF
    // chunks), so the accumulators stay in place from chunk to chunk.
    int chunk = 0;
#pragma unroll 1
    for (int l = 0; l < t - 1; ++l) {
#pragma unroll 1
        for (int cb = 0; cb < chunks_per_block; cb += NBUF, chunk += NBUF)
            static_for<NBUF>([&](auto slot_tag) { run_chunk(slot_tag, chunk + decltype(slot_tag)::value); });
        snapshot(l);
    }
}

// TC tokens per staged chunk, kStateRing chunks per workgroup (one less in flight to cover the
// memory latency); OCC workgroups per CU: grids that exceed one workgroup per CU run two per CU
// with half-size chunks.
// LDS of one state workgroup: the ring, and for NG = 2 the 32 KB behind it for the exchange of
// partial sums at block boundaries.
template <int R, int D, int TC, int NG>
constexpr int state_lds_bytes() { return kStateRing * StateLds<R, D, TC>::BUF + (NG == 2 ? 8 * 16 * 64 * 4 : 0); }

// lds: state_lds_bytes() of workgroup memory, 16-byte aligned; (bid, nblk): this workgroup's
// index among the nblk state workgroups of the launch (dispatch order).
template <int R, int D, int NA, bool SYM, int TC, int NG>
__device__ __forceinline__ void state_workgroup(const float *__restrict__ M8, const bf16_t *__restrict__ V8,
                                                bf16_t *__restrict__ Zg, int n, int b, int t, int units,
                                                unsigned char *lds, int bid, int nblk)
{
    constexpr int NBUF = kStateRing;
    constexpr int BUF_BYTES = StateLds<R, D, TC>::BUF, M_LDS = StateLds<R, D, TC>::M_LDS;
    constexpr int NTHR = kWg * NG;
    constexpr int DMA_PER_CHUNK = (TC * R * 4 + TC * D * 2) / 16 / NTHR;
    constexpr int AG = NA * 4 / (R / 32);
    static_assert(!SYM || NA == 2, "tile deal of the symmetric variant");

    // XCD-aware order: consecutive workgroup ids go to different XCDs, so give each XCD a
    // contiguous range of (unit, group) pairs; the groups of one unit then share one L2.
    int wg = bid;
    if ((nblk & 7) == 0) wg = (bid & 7) * (nblk >> 3) + (bid >> 3);
    constexpr int GROUPS = SYM ? (R / 16) * (R / 16 + 1) / 2 : R / AG;   // workgroups per unit
    const int u = wg / GROUPS, grp = wg % GROUPS;
    if (u >= units || t < 2) return;

    // Prologue shared by both bodies: NBUF-1 chunks in flight, the first one landed.  Chunk
    // indices past the end are clamped: the copies are redundant but keep the in-flight count,
    // and with it the waits, the same in every iteration.
    {
        const int tid = threadIdx.x & 255, wave = tid >> 6;
        const int wg2 = NG == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
        const int chunks = (t - 1) * (b / TC);
        const float *gm = M8 + (size_t)u * n * R;
        const bf16_t *gv = V8 + (size_t)u * n * D;
#pragma unroll
        for (int c = 0; c < NBUF - 1; ++c) {
            const int chunk = min(c, chunks - 1);
            unsigned char *dst = lds + c * BUF_BYTES;
#pragma unroll
            for (int qq = 0; qq < TC * R * 4 / 4096 / NG; ++qq) {
                const int q = qq * NG + wg2;
                dma16(gm + (size_t)chunk * TC * R + (size_t)(q * kWg + tid) * 4,
                      dst + StateLds<R, D, TC>::m_piece(q, wave));
            }
#pragma unroll
            for (int qq = 0; qq < TC * D * 2 / 4096 / NG; ++qq) {
                const int q = qq * NG + wg2;
                dma16(gv + (size_t)chunk * TC * D + (size_t)(q * kWg + tid) * 8,
                      dst + M_LDS + (size_t)(q * kWg + wave * 64) * 16);
            }
        }
        wait_vmem_le<(NBUF - 2) * DMA_PER_CHUNK>();
        __syncthreads();
    }
    state_body<R, D, NA, SYM, TC, NG>(M8, V8, Zg, n, b, t, u, grp, lds);
}

// ------------------------------------------------------------------------------------
// The running prefix state in half precision (r = d = 64, the symmetric deal of state_body with
// NA = 2): m(K) and V arrive as fp16 token octets ([rows/8][64][8], one 1 KB plane per octet), so
// a fragment of phi'(k)^T is four packed multiplies of two LDS operands -- m_j[b'] of the lane's
// column and m_j[a] of its segment's row, each 8 tokens in 16 bytes -- instead of eight
// multiplies and four conversions, and a 64-token chunk is 16 KB of LDS instead of 25.  fp16 has
// three more mantissa bits than the bf16 the same products are rounded to elsewhere; its
// narrow exponent is handled by the scale of the key sketches, one power of two per 128-token
// tile (prep_keys_f16_role): the accumulators hold C Z with C = alpha^2 of the current tile and
// are multiplied by the ratio (a power of two: exact) when the scale changes; the snapshots
// store Z itself, bf16, with the symmetry weights, exactly as state_body does.
//   lds: kStateRing * 16 KB + 2 KB (the unit's scales, at most 512 tiles); (bid, nblk) as for
//   state_workgroup.
// ------------------------------------------------------------------------------------
constexpr int kStateF16Chunk = 64, kStateF16Buf = 2 * kStateF16Chunk * 64 * 2;
constexpr int kStateF16Tiles = 512;             // 128-token tiles per unit, at most
constexpr int kStateF16Lds = kStateRing * kStateF16Buf + kStateF16Tiles * 4;

struct StateOpsF16 {
    f16x8 bfv, av[2], vf[2];
};

template <int R, int D>
__device__ __forceinline__ void state_f16_workgroup(const _Float16 *__restrict__ MKh, const _Float16 *__restrict__ V8h,
                                                    const float *__restrict__ Kscale, bf16_t *__restrict__ Zg,
                                                    int n, int b, int t, int units,
                                                    unsigned char *lds_base, int bid, int nblk)
{
    static_assert(R == 64 && D == 64, "planes of 1 KB, ten workgroups per unit");
    constexpr int TC = kStateF16Chunk, NBUF = kStateRing, CT = 2, NA = 2, SEG = 2, STEPS = TC / 16;
    constexpr int M_BYTES = TC * R * 2, BUF_BYTES = kStateF16Buf, DMA_PER_CHUNK = BUF_BYTES / 16 / kWg;
    constexpr int GROUPS = 10;
    int wg = bid;
    if ((nblk & 7) == 0) wg = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int u = wg / GROUPS, grp = wg % GROUPS;
    if (u >= units || t < 2) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 31, h = lane >> 5;
    int beta = 0, wv = grp * 4 + wave;
    while (wv >= 4 * (beta + 1)) { wv -= 4 * (beta + 1); ++beta; }
    const int a0 = wv * NA * SEG, bcol = 16 * beta + (x & 15);

    // the scales of this unit's 128-token tiles, squared (phi' = m (x) m carries alpha twice)
    float *cs = (float *)(lds_base + NBUF * BUF_BYTES);
    const int tiles = n / 128;
    for (int i = tid; i < tiles && i < kStateF16Tiles; i += kWg) {
        const float al = Kscale[(size_t)u * tiles + i];
        cs[i] = al * al;
    }
    wait_all_memory();

    const unsigned char *gm = (const unsigned char *)(MKh + (size_t)u * n * R);
    const unsigned char *gv = (const unsigned char *)(V8h + (size_t)u * n * D);
    const int chunks = (t - 1) * (b / TC), chunks_per_block = b / TC;
    const uint32_t copy_off = (uint32_t)tid * 16;
    const uint32_t lds0 = lds_address(lds_base);
    auto stage = [&](int slot, int chunk) {          // straight copies: global layout == LDS layout
        const unsigned char *sm = gm + (size_t)chunk * M_BYTES, *sv = gv + (size_t)chunk * M_BYTES;
        const uint32_t dst = lds0 + slot * BUF_BYTES + wave * 1024;
#pragma unroll
        for (int q = 0; q < M_BYTES / 4096; ++q) dma16_sbase(sm + q * 4096, copy_off, dst + q * 4096);
#pragma unroll
        for (int q = 0; q < M_BYTES / 4096; ++q) dma16_sbase(sv + q * 4096, copy_off, dst + M_BYTES + q * 4096);
    };
#pragma unroll
    for (int c = 0; c < NBUF - 1; ++c) stage(c, min(c, chunks - 1));
    wait_vmem_le<(NBUF - 2) * DMA_PER_CHUNK>();
    __syncthreads();

    const unsigned char *lane_b = lds_base + h * 1024 + bcol * 16;
    const unsigned char *lane_a = lds_base + h * 1024 + (a0 + ((lane >> 4) & 1)) * 16;
    const unsigned char *lane_v = lds_base + M_BYTES + h * 1024 + x * 16;
    auto load_ops = [&](auto slot_tag, auto step_tag) {
        constexpr int OFF = decltype(slot_tag)::value * BUF_BYTES + decltype(step_tag)::value * 2048;
        StateOpsF16 o;
        o.bfv = *(const f16x8 *)(lane_b + OFF);
#pragma unroll
        for (int i = 0; i < NA; ++i) o.av[i] = *(const f16x8 *)(lane_a + OFF + i * SEG * 16);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) o.vf[ct] = *(const f16x8 *)(lane_v + OFF + ct * 512);
        return o;
    };

    f32x16 acc[NA][CT];
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < CT; ++j) acc[i][j] = f32x16{0};
    float C = cs[0];

    auto snapshot = [&](int l) {
        bf16_t *z = Zg + ((size_t)u * (t - 1) + l) * R * R * D;
        const float invC = 1.0f / C;
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int a = a0 + i * SEG + gq / 2;
                    const int bq0 = 16 * beta + 8 * (gq % 2) + 4 * h;
                    f32x4 q4;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float wsym = bq0 + j > a ? 2.f : (bq0 + j == a ? 1.f : 0.f);
                        q4[j] = acc[i][ct][4 * gq + j] * (wsym * invC);
                    }
                    *(bf16x4 *)&z[(((size_t)a * (R / 8) + bq0 / 8) * D + 32 * ct + x) * 8 + 4 * h] = cvt4(q4);
                }
    };

    StateOpsF16 ops[2];
    ops[0] = load_ops(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    f16x8 frag = ops[0].bfv * ops[0].av[0];
    auto run_chunk = [&](auto slot_tag, int chunk) {
        constexpr int SLOT = decltype(slot_tag)::value;
        stage((SLOT + NBUF - 1) % NBUF, min(chunk + NBUF - 1, chunks - 1));
        static_for<STEPS>([&](auto s_tag) {
            constexpr int sidx = decltype(s_tag)::value;
            if (sidx == STEPS - 1) {
                wait_vmem_le<(NBUF - 2) * DMA_PER_CHUNK>();
                __builtin_amdgcn_s_barrier();
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (sidx + 1 < STEPS)
                ops[(sidx + 1) & 1] = load_ops(slot_tag, std::integral_constant<int, sidx + 1>{});
            else
                ops[(sidx + 1) & 1] = load_ops(std::integral_constant<int, (SLOT + 1) % NBUF>{},
                                               std::integral_constant<int, 0>{});
            __builtin_amdgcn_sched_group_barrier(0x100, 1 + NA + CT, 0);      // LDS reads first
            const StateOpsF16 &cur = ops[sidx & 1], &nxt = ops[(sidx + 1) & 1];
#pragma unroll
            for (int i = 0; i < NA; ++i) {
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    acc[i][ct] = __builtin_amdgcn_mfma_f32_32x32x16_f16(frag, cur.vf[ct], acc[i][ct], 0, 0, 0);
                frag = i + 1 < NA ? cur.bfv * cur.av[i + 1] : nxt.bfv * nxt.av[0];
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 4 / CT, 0);
                }
            }
        });
    };
    int chunk = 0;
#pragma unroll 1
    for (int l = 0; l < t - 1; ++l) {
#pragma unroll 1
        for (int cb = 0; cb < chunks_per_block; cb += NBUF, chunk += NBUF) {
            static_for<NBUF>([&](auto slot_tag) {
                constexpr int SLOT = decltype(slot_tag)::value;
                if constexpr (SLOT % 2 == 0) {            // a 128-token tile starts: two chunks
                    const float c = cs[min((chunk + SLOT) / 2, kStateF16Tiles - 1)];
                    if (c != C) {                         // wave-uniform
                        const float ratio = c / C;        // powers of two: exact
#pragma unroll
                        for (int i = 0; i < NA; ++i)
#pragma unroll
                            for (int j = 0; j < CT; ++j) acc[i][j] = acc[i][j] * ratio;
                        C = c;
                    }
                }
                run_chunk(slot_tag, chunk + SLOT);
            });
        }
        snapshot(l);
    }
}

template <int R, int D, int NA, bool SYM, int TC, int OCC>
__global__ __launch_bounds__(kWg, OCC) void k_state(const float *__restrict__ M8,
                                               const bf16_t *__restrict__ V8,
                                               bf16_t *__restrict__ Zg, int n, int b, int t,
                                               int units)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[state_lds_bytes<R, D, TC, 1>()];
    state_workgroup<R, D, NA, SYM, TC, 1>(M8, V8, Zg, n, b, t, units, lds, blockIdx.x, gridDim.x);
}

// The symmetric deal with eight waves, two per SIMD (see state_body), one workgroup per CU.
template <int R, int D, int TC>
__global__ __launch_bounds__(2 * kWg, 1) void k_state_two_waves(const float *__restrict__ M8,
                                                                 const bf16_t *__restrict__ V8,
                                                                 bf16_t *__restrict__ Zg, int n, int b, int t,
                                                                 int units)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[state_lds_bytes<R, D, TC, 2>()];
    state_workgroup<R, D, 2, true, TC, 2>(M8, V8, Zg, n, b, t, units, lds, blockIdx.x, gridDim.x);
}

// ------------------------------------------------------------------------------------
// Output kernel.  Workgroup = 128*TT consecutive tokens of one block; wave = TT tiles of 32
// tokens.  All accumulators are D^T-oriented: lane = token, registers = value columns.
// Both phases are software-pipelined inside a wave so that the MFMAs of the next 32x32 item
// are in flight while the VALU works on the current one (x^p, mask, row sums, bf16 packing in
// the in-block phase; the m_i[a] * T_a updates in the cross-block phase).
// ------------------------------------------------------------------------------------
// NONCAUSAL (Section 2.2): no in-block phase, every token takes the cross-block term with the
// one state of its unit (slot 0; the caller passes b = n, t = 2).
// LS (Section 3.1, in-block rule (L R^T)^2): the in-block weights are <m(q_i), m(k_j)>^2 like the
// cross-block ones; Q, K then point to the bf16 rows of m(Q), m(K) (width R instead of D).
// PART splits the work of a token tile over two launches: 0 = everything (one launch);
// 1 = the in-block part only, its unnormalised rows and weight sums left in Pnum / Pden (it
// needs neither the sketches nor the states, so it can run beside the state kernel);
// 2 = the cross-block part, to which what PART 1 left is added at the end (so that its load is
// not in the way of the first chunk of the state), then the division.
// Pnum / Pden layout (private to these two parts, which share this code): per 32-token tile of
// a wave the accumulator registers as they are, [tile][value-column tile][register quad][lane]
// x 16 bytes, and the partial weight sums of the 64 lanes (two per token).  The two launches add
// the same terms as one launch in another order: equal within fp32 rounding, not bit for bit.
// The half-precision state kernel as a launch of its own (any number of units; two workgroups per CU).
template <int R, int D>
__global__ __launch_bounds__(kWg, 2) void k_state_f16(const _Float16 *__restrict__ MKh,
                                                      const _Float16 *__restrict__ V8h,
                                                      const float *__restrict__ Kscale, bf16_t *__restrict__ Zg,
                                                      int n, int b, int t, int units)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[kStateF16Lds];
    state_f16_workgroup<R, D>(MKh, V8h, Kscale, Zg, n, b, t, units, lds, blockIdx.x, gridDim.x);
}

constexpr int kKeyTilesInFlight = 4;
template <int R, int D, int TT, bool LS, int PART>
constexpr int out_lds_bytes()
{
    constexpr int KD = LS ? R : D, TOK_WAVE = 32 * TT, TOK_WG = 4 * TOK_WAVE;
    constexpr int KV = TOK_WAVE * KD * 2 + TOK_WAVE * D * 2;
    constexpr int ZA = 16384 / (R * D);
    constexpr int CROSS = 2 * (ZA * R * D * 2) + 16 * TOK_WG * 2;
    constexpr int INB = kKeyTilesInFlight * KV;
    return PART == 1 ? INB : (PART == 2 ? CROSS : (CROSS > INB ? CROSS : INB));
}

// stage: out_lds_bytes() of workgroup memory, 16-byte aligned; (bid, nblk): this workgroup's
// index among the nblk output workgroups of the launch (dispatch order).
template <int R, int D, int P, int TT, bool DEN, bool NONCAUSAL, bool LS, int PART>
__device__ __forceinline__ void out_workgroup(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                              const bf16_t *__restrict__ V8, const bf16_t *__restrict__ MQ,
                                              const bf16_t *__restrict__ Zg, const bf16_t *__restrict__ Shi,
                                              const bf16_t *__restrict__ Slo, bf16_t *__restrict__ O,
                                              float *__restrict__ Den, float *__restrict__ Pnum,
                                              float *__restrict__ Pden, int n, int b, int t,
                                              unsigned char *stage, int bid, int nblk)
{
    static_assert(PART == 0 || (!NONCAUSAL && (PART == 2 || !DEN)), "the split serves the causal forward call");
    constexpr int KD = LS ? R : D;                        // row width of the in-block score operands
    constexpr int CT = D / 32, KS = KD / 16, RS = R / 16, AT = R / 32;
    constexpr int TOK_WAVE = 32 * TT, TOK_WG = 4 * TOK_WAVE;
    constexpr int KEYT = TOK_WAVE;                        // keys per staged tile = tokens per wave
    constexpr int SUBS = KEYT / 32, IPT = SUBS * TT;      // 32x32 items per staged tile and wave
    constexpr int K_BYTES = KEYT * KD * 2, V_BYTES = KEYT * D * 2;
    constexpr int KV_BYTES = K_BYTES + V_BYTES;           // staged K tile + V tile (16 KB)
    constexpr int NKV = kKeyTilesInFlight;                // key tiles in flight
    constexpr int DMA_KV = KV_BYTES / 16 / kWg;           // copies per thread and tile
    constexpr int ZA = 16384 / (R * D);                   // sketch rows a per staged Z chunk
    constexpr int Z_PER_A = R * D;                        // bf16 elements of Z for one a
    constexpr int Z_CHUNK_BYTES = ZA * Z_PER_A * 2;       // 32 KB
    constexpr int MQ_STEP_BYTES = 16 * TOK_WG * 2;        // m_i[a] of one 16-wide step of a, bf16 [16][TOK_WG]
    static_assert(K_BYTES % (16 * kWg) == 0 && V_BYTES % (16 * kWg) == 0, "whole copies");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int x = lane & 31, h = lane >> 5;
    const int tiles_per_unit = n / TOK_WG;
    // XCD-aware order: consecutive workgroup ids go to different XCDs, so give each XCD a
    // contiguous range of tiles; the workgroups that stream the same Z_l (same unit, same
    // block) then share one L2 and run at about the same time.
    int wg = bid;
    if ((nblk & 7) == 0) wg = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int u = wg / tiles_per_unit;
    // late tiles of a unit first: they carry the cross-block term
    const int tile = tiles_per_unit - 1 - (wg % tiles_per_unit);
    const int i0 = tile * TOK_WG;                         // first token of the workgroup (in unit)
    const int l = i0 / b, jb = l * b;
    const size_t urow = (size_t)u * n;
    const int tok_w0 = i0 + wave * TOK_WAVE;              // first token of this wave

    f32x16 out[TT][CT];
    float den[TT];
    // rows of the workgroup's 32-token tiles in Pnum / Pden
    const size_t ptile0 = (urow + tok_w0) / 32;
    if constexpr (PART == 2) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            den[tt] = Pden[(ptile0 + tt) * 64 + lane];
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) out[tt][ct] = f32x16{0};
        }
    } else {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            den[tt] = 0.f;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) out[tt][ct] = f32x16{0};
        }
    }

    // ---------------- in-block exact weights (Section 3.2) ----------------
    if constexpr (!NONCAUSAL && PART != 2) {
        bf16x8 qfr[TT][KS];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int s = 0; s < KS; ++s)
                qfr[tt][s] = *(const bf16x8 *)&Q[(urow + tok_w0 + 32 * tt + x) * KD + 16 * s + 8 * h];

        // K tile in LDS row by row as in memory, [KEYT keys][KD/8 pieces of 8], so that a copy
        // instruction reads whole rows (a lane per 16-byte piece: 16 cache lines per instruction;
        // one key row per lane would be 64), with the pieces of key j stored at piece ^ swz(j): the
        // A fragments of 8 consecutive keys then fall into different banks.  V tile as
        // [KEYT/8 octets][D][8].  Both filled by direct global->LDS copies.
        constexpr int P8 = KD / 8;                               // 16-byte pieces per key row
        static_assert(P8 == 4 || P8 == 8 || P8 == 16, "swizzle");
        auto swz = [](int key) { return P8 >= 8 ? (key & 7) : ((key >> 1) & 3); };
        const int ntiles_wg = (i0 + TOK_WG - jb) / KEYT;         // tiles staged by the workgroup
        const int ntiles_w = (tok_w0 + TOK_WAVE - jb) / KEYT;    // tiles this wave has keys in
        // (copies: wave-uniform base address in scalar registers + a fixed per-lane offset)
        static_assert(kWg % P8 == 0 && (kWg / P8) % 8 == 0, "key index of a copy slot");
        const uint32_t stage0 = lds_address(stage);
        // copy slot q * kWg + tid = (key q * kWg / P8 + tid / P8, piece tid % P8)
        const uint32_t k_lane = (uint32_t)(((tid / P8) * KD + 8 * ((tid % P8) ^ swz(tid / P8))) * 2);
        const uint32_t v_lane = (uint32_t)tid * 16;
        auto stage_kv = [&](int kt) {
            const int ktc = min(kt, ntiles_wg - 1);              // clamped: keeps the copy count uniform
            const uint32_t dst = stage0 + (kt % NKV) * KV_BYTES + wave * 1024;
            const size_t j0 = urow + jb + (size_t)ktc * KEYT;
            const bf16_t *ksrc = K + j0 * KD, *vsrc = V8 + j0 * D;
#pragma unroll
            for (int q = 0; q < K_BYTES / 16 / kWg; ++q)
                dma16_sbase(ksrc + q * (kWg / P8) * KD, k_lane, dst + q * 4096);
#pragma unroll
            for (int q = 0; q < V_BYTES / 16 / kWg; ++q)
                dma16_sbase(vsrc + q * kWg * 8, v_lane, dst + K_BYTES + q * 4096);
        };

        // Software pipeline over the 32x32 items q of this wave: in one straight-line step the
        // score MFMAs of item q+1 and the P V MFMAs of item q-1 are issued between the VALU work
        // on item q (x^p, mask on the diagonal tile, row sums, bf16 packing).  Score registers
        // and packed weights alternate between two sets by item parity.
        constexpr int PAR = IPT % 2 == 0 ? 1 : 0;          // parity alternates inside a tile only if IPT is even
        f32x16 sc[2];
        bf16x8 pk[2][2];
        bf16x8 kfr[KS], vfr[2][CT];
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {                  // the pipeline's first P V step multiplies these by zero weights
            pk[0][sp] = pk[1][sp] = bf16x8{0};
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) vfr[sp][ct] = bf16x8{0};
        }
        // S^T[key][token] for item q (tile q / IPT, sub-tile, token tile)
        auto score = [&](int q, int jsub, int jtt) {
            const bf16_t *ks = (const bf16_t *)(stage + ((q / IPT) % NKV) * KV_BYTES);
            if (jtt == 0) {
#pragma unroll
                for (int s = 0; s < KS; ++s)
                    kfr[s] = *(const bf16x8 *)&ks[(32 * jsub + x) * KD + 8 * ((2 * s + h) ^ swz(x))];
            }
            f32x16 acc = {0};
#pragma unroll
            for (int s = 0; s < KS; ++s) acc = mfma32(kfr[s], qfr[jtt][s], acc);
            return acc;
        };
        // out^T += V^T P^T for item q with the packed weights pw
        auto apply_pv = [&](int q, int jsub, int jtt, const bf16x8 *pw) {
            const bf16_t *vs = (const bf16_t *)(stage + ((q / IPT) % NKV) * KV_BYTES) + KEYT * KD;
            if (jtt == 0) {                               // fragments serve all token tiles of the sub-tile
#pragma unroll
                for (int sp = 0; sp < 2; ++sp)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct)
                        vfr[sp][ct] = *(const bf16x8 *)&vs[((4 * jsub + 2 * sp + h) * D + 32 * ct + x) * 8];
            }
#pragma unroll
            for (int sp = 0; sp < 2; ++sp)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) out[jtt][ct] = mfma32(vfr[sp][ct], pw[sp], out[jtt][ct]);
        };
        // weights of one item: x^p, causal mask (diagonal tile only), bf16 pack, row sums of the
        // packed values.  The score registers give lane (token, h) the keys
        // 16sp + 8*(e/4) + 4h + e%4; one half-wave swap per register pair turns that into keys
        // 16sp + 8h + e, so that V^T fragments are whole token octets.
        auto weights = [&](auto diag_tag, f32x16 &scv, int jtt, int key0, int tok0, bf16x8 *pw) {
            constexpr bool DIAG = decltype(diag_tag)::value;
            const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float w = LS ? scv[v] * scv[v] : pow_p(scv[v], P);
                if (DIAG) {
                    const int key = key0 + 8 * (v / 4) + 4 * h + (v % 4);
                    w = key <= tok0 + x ? w : 0.f;
                }
                scv[v] = w;
            }
            float dsum = den[jtt];
#pragma unroll
            for (int sp = 0; sp < 2; ++sp) {
                uint4 w = __builtin_bit_cast(uint4, cvt8_from16(scv, 8 * sp));
                dsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.x), ones, dsum, false);
                dsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.y), ones, dsum, false);
                dsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.z), ones, dsum, false);
                dsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.w), ones, dsum, false);
                const auto s0 = __builtin_amdgcn_permlane32_swap(w.x, w.z, false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(w.y, w.w, false, false);
                w.x = s0[0]; w.z = s0[1]; w.y = s1[0]; w.w = s1[1];
                pw[sp] = __builtin_bit_cast(bf16x8, w);
            }
            den[jtt] = dsum;
        };
        // one item: j = position inside the staged tile kt
        auto item = [&](auto diag_tag, auto j_tag, int kt) {
            constexpr int j = decltype(j_tag)::value;
            constexpr int jn = (j + 1) % IPT, jp = (j + IPT - 1) % IPT;
            constexpr int cur = PAR * (j & 1), nxt = PAR * ((j + 1) & 1);
            constexpr int NM = KS + 2 * CT;                       // MFMAs of one step
            constexpr int NV = (P == 8 ? 68 : 52) + (decltype(diag_tag)::value ? 48 : 0);
            const int q = kt * IPT + j;
            __builtin_amdgcn_sched_barrier(0);
            f32x16 sn = score(q + 1, jn / TT, jn % TT);           // garbage past the end, unused
            apply_pv(q - 1 < 0 ? 0 : q - 1, jp / TT, jp % TT, pk[PAR ? nxt : 0]);   // adds zeros at q == 0
            bf16x8 pw[2];
            weights(diag_tag, sc[cur], j % TT, jb + kt * KEYT + 32 * (j / TT), tok_w0 + 32 * (j % TT), pw);
            // LDS reads first, a few VALU operations to cover their latency, then one MFMA per
            // share of the remaining VALU work
            __builtin_amdgcn_sched_group_barrier(0x100, (jn % TT == 0 ? KS : 0) + (jp % TT == 0 ? 2 * CT : 0), 0);
            __builtin_amdgcn_sched_group_barrier(0x002, NV / (NM + 1), 0);
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, NV / (NM + 1), 0);
            }
            sc[PAR ? nxt : 0] = sn;
            pk[PAR ? cur : 0][0] = pw[0];
            pk[PAR ? cur : 0][1] = pw[1];
        };
        // one staged tile: all waves run the same barriers and copies
        auto tile_sync = [&](int kt) {
            // the next tile must have landed for every wave before its first score; the tile
            // before this one is no longer read by anybody, refill its buffer
            wait_vmem_le<(NKV - 3) * DMA_KV>();
            __builtin_amdgcn_s_barrier();
            if (IPT > 1) stage_kv(kt + NKV - 1);
        };
        auto tile_sync_single = [&](int kt) {
            // with one item per tile the previous tile is read right after the barrier: a
            // second barrier separates those reads from the refill
            __builtin_amdgcn_s_barrier();
            stage_kv(kt + NKV - 1);
        };
        auto tile = [&](auto diag_tag, int kt) {
            static_for<IPT>([&](auto j_tag) {
                if (decltype(j_tag)::value == IPT - 1) tile_sync(kt);
                item(diag_tag, j_tag, kt);
                if (IPT == 1) tile_sync_single(kt);
            });
        };

#pragma unroll
        for (int kt = 0; kt < NKV - 1; ++kt) stage_kv(kt);
        wait_vmem_le<(NKV - 2) * DMA_KV>();
        __syncthreads();
        sc[0] = score(0, 0, 0);
        sc[1] = sc[0];
        // Pin the arrival of the Q fragments here.  Left to the compiler, the wait for them sits
        // inside the loop, where it also waits for every key tile copy in flight (the copies
        // are invisible to its counter bookkeeping) and so defeats the ring.
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qfr[tt][s]));
#pragma unroll 1
        for (int kt = 0; kt < ntiles_w - 1; ++kt) tile(std::false_type{}, kt);
        tile(std::true_type{}, ntiles_w - 1);             // the tile that holds this wave's own tokens
        // this wave's keys are exhausted: flush the pending item while its tile is still in LDS
        apply_pv(ntiles_w * IPT - 1, (IPT - 1) / TT, (IPT - 1) % TT, pk[PAR * ((IPT - 1) & 1)]);
#pragma unroll 1
        for (int kt = ntiles_w; kt < ntiles_wg; ++kt) {   // later tiles: only keep the barriers and copies going
            tile_sync(kt);
            if (IPT == 1) tile_sync_single(kt);
        }
        wait_vmem_le<0>();                                // drain the clamped copies
        __syncthreads();
    }

    if constexpr (PART == 1) {
        // leave the unnormalised rows and the weight sums for the second launch
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            Pden[(ptile0 + tt) * 64 + lane] = den[tt];      // per lane: the two halves of a wave hold different keys
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq)
                    *(f32x4 *)&Pnum[(((ptile0 + tt) * CT + ct) * 4 + gq) * 256 + lane * 4] =
                        f32x4{out[tt][ct][4 * gq], out[tt][ct][4 * gq + 1], out[tt][ct][4 * gq + 2],
                              out[tt][ct][4 * gq + 3]};
        }
        return;
    }

    // ---------------- cross-block term phi'(Q_l) Z_l (Section 3.1) ----------------
    bool cross = l > 0;
    if constexpr (NONCAUSAL) cross = t > 1;               // always true there; kept a run-time branch on purpose
    if (cross) {
        bf16x8 mfr[TT][RS];                               // B operands: m(q_i), k index = b'
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int s = 0; s < RS; ++s)
                mfr[tt][s] = *(const bf16x8 *)&MQ[(urow + tok_w0 + 32 * tt + x) * R + 16 * s + 8 * h];

        // numerator: phi'(q_i)^T Z_l with phi'(q_i) = m_i (x) m_i expanded in registers.  For
        // sketch row a and 16-wide step s the B operand is B[k = b'][j = token] = m_i[a] * m_i[b']
        // (12 VALU operations per fragment, each feeding CT MFMAs that accumulate straight into
        // `out`), the A operand a fragment of Z_l[a] read from LDS.
        f32x8 mb[TT][RS];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int s = 0; s < RS; ++s)
#pragma unroll
                for (int e = 0; e < 8; ++e) mb[tt][s][e] = (float)mfr[tt][s][e];

        const bf16_t *zsrc = Zg + ((size_t)u * (t - 1) + (NONCAUSAL ? 0 : l - 1)) * R * R * D;
        const uint32_t stage0 = lds_address(stage);
        constexpr int NCHUNK = R / ZA;
        constexpr int BUF_BYTES = Z_CHUNK_BYTES;
        static_assert(PART == 1 || 2 * BUF_BYTES + MQ_STEP_BYTES <= out_lds_bytes<R, D, TT, LS, PART>(), "stage size");
        // m_i[a] for the 16 sketch rows a of one 16-wide step, bf16 [16][TOK_WG] behind the two Z
        // buffers, written from the fp32 copies of the B operands when the chunks reach the step:
        // lane (x, h) holds entries a % 16 = 8 h + e of its tokens.  Every wave writes and reads
        // only its own tokens, in program order: no barrier is involved.  (A second read of
        // m(Q) from memory, 8 bytes of every row per chunk, cost an L1 access per lane and chunk:
        // a tenth of this kernel's time.)
        constexpr int PER = 16 / ZA;                         // chunks per step
        static_assert(16 % ZA == 0, "whole chunks per step");
        uint16_t *mq_step = (uint16_t *)(stage + 2 * BUF_BYTES);
        // Z is stored with the symmetry weights baked in (see k_state): for sketch row a only
        // b' >= 16 * (a / 16) contributes, i.e. 16-wide steps s >= s0 = a / 16 and octets >= 2 s0.
        // All rows of a chunk share s0.
        static_assert(16 % ZA == 0, "one s0 per chunk");
        // The needed part of a chunk is copied in 1 KB pieces (one per wave and copy): piece c
        // covers columns 64 * (c % DW).. of octet 2 s0 + c / (DW * ZA) of row (c / DW) % ZA;
        // wave w issues the pieces w, w + 4, ...
        constexpr int DW = D / 64;
        constexpr int KPA = R * D / 2048;                    // copies per wave and row a, at most
        static_assert(DW >= 1 && KPA >= 1 && (ZA * DW) % 2 == 0, "piece enumeration");
        auto z_ncopy = [&](int chunk) { return (R / 8 - 2 * (chunk * ZA / 16)) * ZA * DW / 4; };
        auto stage_z_k = [&](int buf, int chunk, int k) {
            const int c = wave + 4 * k;
            const int off = (((c / DW) % ZA) * (R / 8) + 2 * (chunk * ZA / 16) + c / (DW * ZA)) * D +
                            (c % DW) * 64;                   // 16-byte units inside the chunk
            dma16_sbase(zsrc + (size_t)chunk * ZA * Z_PER_A + (size_t)off * 8, (uint32_t)lane * 16,
                        stage0 + buf * BUF_BYTES + off * 16);
        };
        auto store_mq = [&](auto s_tag) {
            constexpr int S = decltype(s_tag)::value;
            if constexpr (S < RS) {
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        mq_step[(8 * h + e) * TOK_WG + wave * TOK_WAVE + 32 * tt + x] =
                            (uint16_t)(__float_as_uint(mb[tt][S][e]) >> 16);      // exact: mb holds bf16 values
            }
        };
        auto gen = [&](float ma, const f32x8 &mbv) {
            f32x8 pr;
#pragma unroll
            for (int e = 0; e < 8; ++e) pr[e] = ma * mbv[e];
            return cvt8(pr);
        };
        for (int k = 0; k < z_ncopy(0); ++k) stage_z_k(0, 0, k);
        // denominator: m_i^T S m_i with S = prefix of m_j m_j^T, hi + lo operands
        {
            const size_t sbase = ((size_t)u * (t - 1) + (NONCAUSAL ? 0 : l - 1)) * R * R;
#pragma unroll
            for (int at = 0; at < AT; ++at) {
                f32x16 td[TT];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) td[tt] = f32x16{0};
#pragma unroll
                for (int s = 0; s < RS; ++s) {
                    const size_t off = sbase + ((size_t)(2 * s + h) * R + 32 * at + x) * 8;
                    const bf16x8 s_hi = *(const bf16x8 *)&Shi[off], s_lo = *(const bf16x8 *)&Slo[off];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) {
                        td[tt] = mfma32(s_hi, mfr[tt][s], td[tt]);
                        td[tt] = mfma32(s_lo, mfr[tt][s], td[tt]);
                    }
                }
                // m_i[a] for the rows a = 32 at + 8 gq + 4 h + j this lane holds of td: they sit in
                // the B operands already, half of them in the other half-wave (one swap per pair)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        const uint4 w = __builtin_bit_cast(uint4, mfr[tt][2 * at + s2]);
                        const auto s0 = __builtin_amdgcn_permlane32_swap(w.x, w.z, false, false);
                        const auto s1 = __builtin_amdgcn_permlane32_swap(w.y, w.w, false, false);
                        // lane h = 0: s0[0], s1[0] = elements 0..3, s0[1], s1[1] = elements 8..11 of the 16;
                        // lane h = 1: elements 4..7 and 12..15
                        const uint32_t pr[4] = {s0[0], s1[0], s0[1], s1[1]};
#pragma unroll
                        for (int g2 = 0; g2 < 2; ++g2)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const uint32_t word = pr[2 * g2 + j / 2];
                                const float mv = __uint_as_float((j & 1) ? (word & 0xffff0000u) : (word << 16));
                                den[tt] += mv * td[tt][4 * (2 * s2 + g2) + j];
                            }
                    }
            }
        }

        store_mq(std::integral_constant<int, 0>{});
        wait_all_memory();
        __syncthreads();
        auto chunk_iter = [&](auto s0_tag, int chunk) {
            const int buf = chunk & 1;
            // the next chunk's copies are issued a few per row a inside the loop below: issued
            // back to back they stall this wave on the memory pipeline's queue
            const int n_copies = chunk + 1 < NCHUNK ? z_ncopy(chunk + 1) : 0;
            const bf16_t *zc = (const bf16_t *)(stage + buf * BUF_BYTES);
            const uint16_t *mqs = mq_step + (chunk % PER) * ZA * TOK_WG;
            auto run_chunk = [&](auto s0_tag) {
                constexpr int S0 = decltype(s0_tag)::value;  // first 16-wide step with b' >= a
                constexpr int NS = RS - S0;
                bf16x8 zf[2][CT][RS];                        // fragments of Z[a], ping-pong over a
                float ma[2][TT];                             // m_i[a] of this lane's tokens
                auto load_a = [&](int ai) {
                    const bf16_t *za = zc + ai * Z_PER_A;
#pragma unroll
                    for (int s = S0; s < RS; ++s)
#pragma unroll
                        for (int ct = 0; ct < CT; ++ct)
                            zf[ai & 1][ct][s] = *(const bf16x8 *)&za[((2 * s + h) * D + 32 * ct + x) * 8];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        ma[ai & 1][tt] =
                            __uint_as_float((uint32_t)mqs[ai * TOK_WG + wave * TOK_WAVE + 32 * tt + x] << 16);
                };
                load_a(0);
                bf16x8 frag = gen(ma[0][0], mb[0][S0]);
#pragma unroll
                for (int ai = 0; ai < ZA; ++ai) {
#pragma unroll
                    for (int c = 0; c < KPA; ++c)
                        if (ai * KPA + c < n_copies) stage_z_k(buf ^ 1, chunk + 1, ai * KPA + c);
                    __builtin_amdgcn_sched_barrier(0);
                    if (ai + 1 < ZA) load_a(ai + 1);
#pragma unroll
                    for (int it = 0; it < NS * TT; ++it) {
                        const int s = S0 + it / TT, tt = it % TT, itn = it + 1;
                        bf16x8 nxt = frag;
                        if (itn < NS * TT) nxt = gen(ma[ai & 1][itn % TT], mb[itn % TT][S0 + itn / TT]);
                        else if (ai + 1 < ZA) nxt = gen(ma[(ai + 1) & 1][0], mb[0][S0]);
#pragma unroll
                        for (int ct = 0; ct < CT; ++ct)
                            out[tt][ct] = mfma32(zf[ai & 1][ct][s], frag, out[tt][ct]);
#pragma unroll
                        for (int ct = 0; ct < CT; ++ct) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x002, 12 / CT, 0);
                        }
                        frag = nxt;
                    }
                }
            };
            run_chunk(s0_tag);
            wait_all_memory();
            __syncthreads();
        };
        // one loop per step (the chunks come in the order of their first step s0), each with a
        // single body, so that the accumulators are carried by simple loops; between two of them
        // the next step's m_i[a] go to the table
        static_assert(NCHUNK == RS * PER, "chunks per step");
        static_for<RS>([&](auto s0_tag) {
            constexpr int S0 = decltype(s0_tag)::value;
#pragma unroll 1
            for (int chunk = S0 * PER; chunk < (S0 + 1) * PER; ++chunk) chunk_iter(s0_tag, chunk);
            store_mq(std::integral_constant<int, S0 + 1>{});
        });
    }

    if constexpr (PART == 2) {
        // the in-block part, left by the first launch
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const f32x4 q4 = *(const f32x4 *)&Pnum[(((ptile0 + tt) * CT + ct) * 4 + gq) * 256 + lane * 4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[tt][ct][4 * gq + j] += q4[j];
                }
    }
    // ---------------- normalise and store (Section 3: divide by 1 + sum of weights) ----------------
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const float total = den[tt] + __shfl_xor(den[tt], 32);   // the two halves hold different keys / rows
        const float inv = 1.0f / (1.0f + total);
        const size_t row = urow + tok_w0 + 32 * tt + x;
        if (DEN && h == 0) Den[row] = 1.0f + total;        // kept for the backward pass
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                f32x4 q4 = {out[tt][ct][4 * gq] * inv, out[tt][ct][4 * gq + 1] * inv,
                            out[tt][ct][4 * gq + 2] * inv, out[tt][ct][4 * gq + 3] * inv};
                *(bf16x4 *)&O[row * D + 32 * ct + 8 * gq + 4 * h] = cvt4(q4);
            }
    }
}

template <int R, int D, int P, int TT, bool DEN, bool NONCAUSAL = false, bool LS = false, int PART = 0>
__global__ __launch_bounds__(kWg, 2) void k_out(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                const bf16_t *__restrict__ V8,
                                                const bf16_t *__restrict__ MQ,
                                                const bf16_t *__restrict__ Zg,
                                                const bf16_t *__restrict__ Shi,
                                                const bf16_t *__restrict__ Slo, bf16_t *__restrict__ O,
                                                float *__restrict__ Den, float *__restrict__ Pnum,
                                                float *__restrict__ Pden, int n, int b, int t)
{
    __shared__ __attribute__((aligned(16))) unsigned char stage[out_lds_bytes<R, D, TT, LS, PART>()];
    out_workgroup<R, D, P, TT, DEN, NONCAUSAL, LS, PART>(Q, K, V8, MQ, Zg, Shi, Slo, O, Den, Pnum, Pden, n, b, t,
                                                         stage, blockIdx.x, gridDim.x);
}

// The state kernel in one launch with everything that does not depend on its results: the
// in-block part of the output kernel (reads Q, K, V only), the sketch of the query rows and the
// scan of the denominator partials (both first needed by the cross-block part afterwards).
// They stall on different things: a state workgroup is one wave per SIMD that waits on its LDS
// operands between MFMAs, the in-block part is bound by the vector work on its score tiles, the
// query sketch by memory.  Side by side on a CU each fills what the others leave idle.  The
// first n_state workgroups (dispatched first: one per CU as long as there are at most as many
// as CUs) run the state kernel in its two-per-CU form, the next n_den the scan, and the rest
// alternate: `ratio` 128 * TT token tiles of the in-block part, then one part of the sketch.
struct BesideStates {
    const bf16_t *Q, *K, *G;                   // rows as given; sketch matrices [d][r] row-major
    float *Pnum, *Pden;                        // in-block part out
    bf16_t *MQ;                                // query sketch out
    const float *Spart;                        // scan in
    bf16_t *Shi, *Slo;                         // scan out
    int heads, per_head, tiles_per_wg, parts_per_block, parts_per_unit;
    int n_state, n_den, n_tiles, ratio;        // workgroups per role; in-block tiles between two sketch parts
    size_t g_len;
    const _Float16 *V8h;                       // half-precision state kernel: value octets, key scales
    const float *Kscale;                       // one per 128-token tile
};

// F16: the state role runs state_f16_workgroup (M8 then holds the fp16 key sketches).
template <int R, int D, int P, int TT, bool F16>
__global__ __launch_bounds__(kWg, 2) void k_state_and_in_block(const float *__restrict__ M8,
                                                               const bf16_t *__restrict__ V8,
                                                               bf16_t *__restrict__ Zg, int units, int n, int b,
                                                               int t, BesideStates a)
{
    constexpr int TC = 32;
    constexpr int S_BYTES = F16 ? kStateF16Lds : state_lds_bytes<R, D, TC, 1>();
    constexpr int O_BYTES = out_lds_bytes<R, D, TT, false, 1>();
    constexpr int BYTES = S_BYTES > O_BYTES ? S_BYTES : O_BYTES;
    static_assert(sizeof(PrepLds<D, R>) <= BYTES, "the sketch role fits the same allocation");
    __shared__ __attribute__((aligned(16))) unsigned char lds[BYTES];
    int bid = blockIdx.x;
    if (bid < a.n_state) {
        if constexpr (F16)
            state_f16_workgroup<R, D>((const _Float16 *)M8, a.V8h, a.Kscale, Zg, n, b, t, units, lds, bid, a.n_state);
        else
            state_workgroup<R, D, 2, true, TC, 1>(M8, V8, Zg, n, b, t, units, lds, bid, a.n_state);
        return;
    }
    bid -= a.n_state;
    if (bid < a.n_den) {
        constexpr int PER_UNIT = R * R / kWg;
        den_scan_workgroup<R>(a.Spart, a.Shi, a.Slo, t, a.parts_per_block, a.parts_per_unit, bid / PER_UNIT,
                              bid % PER_UNIT, (bf16_t *)lds);
        return;
    }
    bid -= a.n_den;
    const int period = a.ratio + 1;
    if (bid % period == a.ratio) {
        const size_t tok_wg0 = (size_t)(bid / period) * a.tiles_per_wg * 128;
        const int u = (int)(tok_wg0 / n);
        const bf16_t *g = a.G + (a.per_head ? (size_t)(u % a.heads) * a.g_len : 0);
        prep_sketch_role<D, R, true>(*reinterpret_cast<PrepLds<D, R> *>(lds), a.Q, g, tok_wg0, a.tiles_per_wg, a.MQ,
                                     nullptr, nullptr);
    } else {
        out_workgroup<R, D, P, TT, false, false, false, 1>(a.Q, a.K, V8, nullptr, nullptr, nullptr, nullptr, nullptr,
                                                           nullptr, a.Pnum, a.Pden, n, b, t, lds,
                                                           (bid / period) * a.ratio + bid % period, a.n_tiles);
    }
}

// ------------------------------------------------------------------------------------
// Learned sketches (Algorithm 2): m(x) comes from the general fp32 sketch kernel as row-major
// fp32 [rows][R]; these two kernels put it into the layouts the state and output kernels read.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWg) void k_m_to_bf16(const float *__restrict__ M, bf16_t *__restrict__ MQ,
                                                   size_t count)
{
    const size_t i = ((size_t)blockIdx.x * kWg + threadIdx.x) * 4;
    if (i + 3 < count) {
        const f32x4 v = *(const f32x4 *)&M[i];
        *(bf16x4 *)&MQ[i] = cvt4(v);
    } else {
        for (size_t e = i; e < count; ++e) MQ[e] = f32_to_bf16(M[e]);
    }
}

// One workgroup per part of `tokens` consecutive tokens of one unit: m(K) rows -> token octets
// [n/8][2][R][4] fp32, and the part's S = m^T m (R x R, fp32) for the denominator scan.
// (MT: fp32 rows from the general sketch kernel, or bf16 rows that are the sketch already, p = 2.)
template <int R, typename MT = float>
__global__ __launch_bounds__(kWg) void k_m_to_octets_and_partials(const MT *__restrict__ M,
                                                                  float *__restrict__ MK8,
                                                                  float *__restrict__ Spart, int tokens)
{
    constexpr int TCH = 64, PER = R * R / kWg;            // staged tokens; S entries per thread
    __shared__ float ms[TCH][R + 1];
    const int tid = threadIdx.x;
    const size_t row0 = (size_t)blockIdx.x * tokens;      // parts tile the rows of all units in order
    float acc[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) acc[q] = 0.f;
    for (int t0 = 0; t0 < tokens; t0 += TCH) {
        __syncthreads();
        for (int idx = tid; idx < TCH * R; idx += kWg) {
            const int tk = idx / R, c = idx % R;
            const float v = load_f(M, (row0 + t0 + tk) * R + c);
            ms[tk][c] = v;
            const size_t tok = row0 + t0 + tk;            // octet layout: ((tok/8 * 2 + (tok%8)/4) * R + c) * 4 + tok%4
            MK8[((tok / 8 * 2 + (tok % 8) / 4) * R + c) * 4 + tok % 4] = v;
        }
        __syncthreads();
        // entry e = q * kWg + tid of S: column c = tid % R for every q, row a = q * (kWg / R) + tid / R
        // (the same row for the whole wave: a broadcast read)
        const int c = tid % R, a0 = tid / R;
        for (int tk = 0; tk < TCH; ++tk) {
            const float mc = ms[tk][c];
#pragma unroll
            for (int q = 0; q < PER; ++q) acc[q] += ms[tk][q * (kWg / R) + a0] * mc;
        }
    }
    float *out = Spart + (size_t)blockIdx.x * R * R;
#pragma unroll
    for (int q = 0; q < PER; ++q) out[q * kWg + tid] = acc[q];
}

// ------------------------------------------------------------------------------------
// Learned sketches on MFMA (Algorithm 2 with d = 64 or 128; degree 4: m(x) =
// sqrt(r) tanh(f1(x) * f2(x) / sqrt(r)), degree 8: the same node once more on two such sketches),
// f = the four-layer network of Appendix D.
// Everything is "transposed": accumulators hold [feature][token] (lane = token), so a layer's
// output registers are the next layer's B operand after a bf16 conversion; the weights are
// the A operands, pre-arranged by k_learned_prep so that every fragment is one 16-byte read
// and the contraction order matches the accumulator register order.  Layer normalisation is
// folded into the weights:  LN(a) W = (a (g . W) - mean (sum_k g_k W_k)) / sigma + b W.  For
// the input layer the mean / sigma terms ride on a fifth contraction step (hi + lo bf16 pairs),
// for the second one they are applied after the product has been accumulated over all hidden
// chunks, together with the sums of h and h^2.  Hidden width 8r is walked in chunks of 32;
// the weights of a chunk (8 KB) stream through a ring of LDS slots.
// ------------------------------------------------------------------------------------
constexpr int kLsSlotBytes = 8192;     // one chunk at d = 64: [W1' | W2'] or [W3 | W4], second part at +4096
// d = 128: W1' is eight 1 KB k-steps, so the second part sits at +8192 and a slot is 16 KB
__host__ __device__ constexpr int ls_slot_bytes(int d) { return d == 64 ? kLsSlotBytes : 2 * kLsSlotBytes; }
constexpr int kLsRing = 4;

__device__ __forceinline__ float gelu_fast(float x)
{
    // tanh form: 0.5 x (1 + tanh(u)), u = sqrt(2/pi) (x + 0.044715 x^3)  =  x - x / (1 + exp(2u))
    const float e = __builtin_amdgcn_exp2f(x * (2.3022082f + 0.10294324f * x * x));   // exp(2u) as 2^(.)
    return x - x * __builtin_amdgcn_rcpf(1.0f + e);
}

// The same function without the two quarter-rate instructions: gelu(x) = x s(x), s - 1/2 odd in x;
// s(x) ~ 1/2 + x P(x^2) with a degree-5 P fitted (minimax in x s) on |x| <= 3.5, x clamped to
// that range before P (s(3.5) = 0.99984).  |gelu_poly - gelu| <= 2.8e-4 for |x| <= 3.5 and
// <= 1.6e-4 |x| beyond: below the fp16 rounding of the activations it feeds and below the
// distance between the tanh form and the erf form of gelu (4.7e-4).  Nine full-rate
// instructions against six + exp2 + rcp (the forward network kernel is bound by exactly these).
__device__ __forceinline__ float gelu_poly(float x)
{
    const float xc = __builtin_amdgcn_fmed3f(x, -3.5f, 3.5f);
    const float x2 = xc * xc;
    float p = -7.189494226622628e-07f;
    p = fmaf(p, x2, 3.4920682082884014e-05f);
    p = fmaf(p, x2, -0.0007207939634099603f);
    p = fmaf(p, x2, 0.008435080759227276f);
    p = fmaf(p, x2, -0.06395040452480316f);
    p = fmaf(p, x2, 0.3973534405231476f);
    return x * fmaf(xc, p, 0.5f);
}

__device__ __forceinline__ float tanh_fast(float y)
{
    const float e = __builtin_amdgcn_exp2f(2.8853900f * y);                           // exp(2y)
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + e);
}

// Operand type of the network layers: fp16.  With bf16 operands the rounding of every layer's
// inputs to 8 mantissa bits adds up: at degree 8 (two levels of networks) to the whole tolerance
// of the path, at degree 4 to two thirds of it once the gradients go through the same sketches.
// fp16 has 11 bits; the weights are bf16 values, exact in fp16 unless below 2^-14; activations
// are layer-normalised rows and gelu outputs, far inside +-65504 for any network with
// O(1)-scaled weights -- beyond that range they would overflow.  (LsOp<false> keeps the bf16
// variant of the same code.)
constexpr bool kLsHalf = true;
template <bool HALF>
struct LsOp;
template <>
struct LsOp<false> {
    typedef bf16x8 v8;
    typedef __bf16 elem;
    __device__ static __forceinline__ v8 cvt(f32x8 x) { return cvt8(x); }
    __device__ static __forceinline__ f32x16 mfma(v8 a, v8 b, f32x16 c) { return mfma32(a, b, c); }
    __device__ static __forceinline__ uint16_t bits(float v) { return f32_to_bf16(v); }
    __device__ static __forceinline__ float rounded(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};
template <>
struct LsOp<true> {
    typedef f16x8 v8;
    typedef _Float16 elem;
    __device__ static __forceinline__ v8 cvt(f32x8 x) { return __builtin_convertvector(x, f16x8); }
    __device__ static __forceinline__ f32x16 mfma(v8 a, v8 b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ uint16_t bits(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }
    __device__ static __forceinline__ float rounded(float v) { return (float)(_Float16)v; }
};
template <class Op>
__device__ __forceinline__ typename Op::v8 ls_cvt_from16(const f32x16 &v, int first)
{
    f32x8 t;
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = v[first + e];
    return Op::cvt(t);
}

// Parameter blob of one network of input width win (64 for the networks on x, R for the two
// second-level ones of degree 8): g1, b1, W1 [win][8R], g2, b2, W2 [8R][R], W3 [R][8R], W4 [8R][R].
template <int R, int D_IN = 64>
struct LearnedNet {
    static constexpr int HID = 8 * R, NCH = HID / 32, D = D_IN;
    __host__ __device__ static constexpr size_t len(int win)
    {
        return 2 * (size_t)win + (size_t)win * HID + 2 * HID + 3 * (size_t)HID * R;
    }
    // offset of network `net` in a parameter set of degree p (Appendix D order: the p / 2 networks
    // on x, then the ones on sketches) and its input width
    __host__ __device__ static constexpr int win_of(int net, int p) { return net < p / 2 ? D : R; }
    __host__ __device__ static constexpr size_t offset_of(int net, int p)
    {
        return net < p / 2 ? net * len(D) : (p / 2) * len(D) + (net - p / 2) * len(R);
    }
    const bf16_t *g1, *b1, *W1, *g2, *b2, *W2, *W3, *W4;
    __device__ LearnedNet(const bf16_t *P, int win)
    {
        g1 = P; b1 = g1 + win; W1 = b1 + win; g2 = W1 + (size_t)win * HID; b2 = g2 + HID; W2 = b2 + HID;
        W3 = W2 + (size_t)HID * R; W4 = W3 + (size_t)R * HID;
    }
};

// Slot (net, phase, chunk) of the weight stream of one parameter set; grid (2 * (P - 2) * NCH, sets).
//   phase 0: [0, 4 KB)  W1' fragments: k-step s < 4, hidden row i, half h, e: k = 16 s + 8 h + e,
//                       value bf16(g1[k] W1[k][32 ch + i]); for the networks on sketches (degree 8)
//                       k runs in accumulator row order like W3's feature below, zero past R
//            [4 KB, ..) W2' fragments: out tile ot, k-step s < 2, out row i, half h, e:
//                       hidden = 32 ch + 16 s + 8 (e / 4) + 4 h + e % 4 (accumulator row order),
//                       value bf16(g2[hidden] W2[hidden][32 ot + i])
//   phase 1: [0, 4 KB)  W3 fragments: k-step t < R / 16, hidden row i, half h, e:
//                       feature = 32 (t / 2) + 16 (t % 2) + 8 (e / 4) + 4 h + e % 4
//            [4 KB, ..) W4 fragments, arranged like W2' without the scale.
template <int R, int P_DEG = 4, int D_IN = 64>
__global__ __launch_bounds__(kWg) void k_learned_prep(const bf16_t *__restrict__ P, size_t p_len,
                                                      bf16_t *__restrict__ LW, float *__restrict__ C1,
                                                      float *__restrict__ LVp)
{
    using Net = LearnedNet<R, D_IN>;
    using Op = LsOp<kLsHalf>;
    constexpr int NCH = Net::NCH, HID = Net::HID, D = Net::D, NETS = P_DEG - 2;
    constexpr int SLOT = ls_slot_bytes(D), PART_ELEMS = SLOT / 4;      // bf16 / fp16 entries of one half of a slot
    __shared__ float red[2][kWg];
    const int q = blockIdx.x, set = blockIdx.y, tid = threadIdx.x;
    const int net = q / (2 * NCH), phase = (q / NCH) % 2, ch = q % NCH;
    const int win = Net::win_of(net, P_DEG);
    const bool on_sketch = net >= P_DEG / 2;
    const Net nt(P + (size_t)set * p_len + Net::offset_of(net, P_DEG), win);
    bf16_t *slot = LW + ((size_t)set * 2 * NETS * NCH + q) * (SLOT / 2);
    for (int idx = tid; idx < SLOT / 2; idx += kWg) {
        float v = 0.f;
        const int part = idx / PART_ELEMS, r2 = idx % PART_ELEMS;
        const int i = (r2 % 512) / 16, h = (r2 / 8) % 2, e = r2 % 8, blk = r2 / 512;
        const int perm = 8 * (e / 4) + 4 * h + e % 4;           // accumulator row order inside 16
        if (phase == 0 && part == 0) {
            const int k = on_sketch ? 32 * (blk / 2) + 16 * (blk % 2) + perm : 16 * blk + 8 * h + e;
            if (k < win && blk < D / 16) v = bf16_to_f32(nt.g1[k]) * bf16_to_f32(nt.W1[(size_t)k * HID + 32 * ch + i]);
        } else if (phase == 0) {
            if (blk < 2 * (R / 32)) {
                const int ot = blk / 2, sstep = blk % 2, hid = 32 * ch + 16 * sstep + perm;
                v = bf16_to_f32(nt.g2[hid]) * bf16_to_f32(nt.W2[(size_t)hid * R + 32 * ot + i]);
            }
        } else if (part == 0) {
            if (blk < R / 16) {
                const int feat = 32 * (blk / 2) + 16 * (blk % 2) + perm;
                v = bf16_to_f32(nt.W3[(size_t)feat * HID + 32 * ch + i]);
            }
        } else {
            if (blk < 2 * (R / 32)) {
                const int ot = blk / 2, sstep = blk % 2, hid = 32 * ch + 16 * sstep + perm;
                v = bf16_to_f32(nt.W4[(size_t)hid * R + 32 * ot + i]);
            }
        }
        slot[idx] = Op::bits(v);
    }
    if (phase != 0) return;
    // constants of the folded layer normalisations for the 32 hidden units of this chunk:
    //   C1 [set][net][NCH][32] fp32: c1 = sum_k b1[k] W1[k][.]  (the accumulators of the input layer start there)
    //   LVp [set][net][NCH][2][R] fp32: this chunk's part of s2 = sum_hid (g2 W2 as stored), c2 = sum_hid b2 W2
    {
        const int i = tid & 31, kp = tid >> 5, hid = 32 * ch + i;
        float c1 = 0.f;
        for (int k = (D / 8) * kp; k < (D / 8) * (kp + 1); ++k)
            if (k < win) c1 += bf16_to_f32(nt.b1[k]) * bf16_to_f32(nt.W1[(size_t)k * HID + hid]);
        red[0][tid] = c1;
        __syncthreads();
        if (tid < 32) {
            c1 = 0.f;
            for (int kk = 0; kk < kWg / 32; ++kk) c1 += red[0][32 * kk + tid];
            C1[(((size_t)set * NETS + net) * NCH + ch) * 32 + tid] = c1;
        }
        __syncthreads();
    }
    {
        constexpr int GR = kWg / R, PER = 32 / GR;              // hidden units of the chunk per thread
        const int out = tid % R, hp = tid / R;
        float s2 = 0.f, c2 = 0.f;
        for (int hh = 0; hh < PER; ++hh) {
            const int hid = 32 * ch + hp * PER + hh;
            const float w = bf16_to_f32(nt.W2[(size_t)hid * R + out]);
            s2 += Op::rounded(bf16_to_f32(nt.g2[hid]) * w);
            c2 += bf16_to_f32(nt.b2[hid]) * w;
        }
        red[0][tid] = s2;
        red[1][tid] = c2;
        __syncthreads();
        if (tid < R) {
            s2 = c2 = 0.f;
            for (int g = 0; g < GR; ++g) { s2 += red[0][g * R + tid]; c2 += red[1][g * R + tid]; }
            float *o = LVp + (((size_t)set * NETS + net) * NCH + ch) * 2 * R;
            o[tid] = s2;
            o[R + tid] = c2;
        }
    }
}

// Workgroup = 256 consecutive tokens of one unit, 8 / TT waves with TT tiles of 32 tokens each.
//   QSIDE: writes m(x) as bf16 rows [rows][R].
//   key side: the last layer runs with the operand roles swapped, so that lanes hold sketch
//   columns and registers tokens; writes the token octets [rows/8][2][R][4] fp32 and the
//   workgroup's S = m^T m (R x R fp32, from the bf16 m like the random-sketch kernel does).
// P_DEG = 8: three nodes -- networks 0, 1 and 2, 3 on x, then 4 on the first node's sketch and 5
// on the second's (their inputs are the accumulator registers of the nodes, normalised in place:
// no layout change, their first-layer weights are arranged in that register order).
template <int R, bool QSIDE, int TT, int P_DEG = 4, int D_IN = 64>
__global__ __launch_bounds__(512 / TT, 1) void k_learned_sketch(const bf16_t *__restrict__ X,
                                                                const bf16_t *__restrict__ LW,
                                                                const float *__restrict__ C1,
                                                                const float *__restrict__ LVp,
                                                                bf16_t *__restrict__ M_rm,
                                                                float *__restrict__ M8,
                                                                float *__restrict__ Spart, int n, int heads,
                                                                int per_head)
{
    using Net = LearnedNet<R, D_IN>;
    using Op = LsOp<kLsHalf>;
    typedef typename Op::v8 op8;
    constexpr int NCH = Net::NCH, HID = Net::HID, D = D_IN, OT = R / 32, KS = D / 16, RS = R / 16;
    constexpr int SLOT = ls_slot_bytes(D), PART1 = SLOT / 2;  // bytes of a slot; offset of its second part
    constexpr int NW = 8 / TT, NTHR = 64 * NW;             // waves, threads
    constexpr int NETS = P_DEG - 2;
    constexpr int QN = 2 * NETS * NCH;                     // slots of the weight stream
    constexpr int DMA = SLOT / 16 / NTHR;          // copies per thread and slot
    static_assert(NW * 32 * 32 * 4 <= kLsRing * SLOT, "the reduction of S reuses the ring");
    __shared__ __attribute__((aligned(16))) unsigned char ring[kLsRing * SLOT];
    __shared__ __attribute__((aligned(16))) float c1s[NETS * NCH * 32];
    __shared__ __attribute__((aligned(16))) float lv[NETS * 2 * R];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 31, h = lane >> 5;
    const size_t row0 = (size_t)blockIdx.x * 256;
    const int set = per_head ? (int)((row0 / n) % heads) : 0;
    const unsigned char *stream = (const unsigned char *)(LW + (size_t)set * QN * (SLOT / 2));
    const uint32_t ring0 = lds_address(ring);
    auto stage = [&](int q) {
        const int qc = min(q, QN - 1);                     // clamped: keeps the copy count uniform
        const uint32_t dst = ring0 + (q % kLsRing) * SLOT + wave * 1024;
#pragma unroll
        for (int c = 0; c < DMA; ++c)
            dma16_sbase(stream + (size_t)qc * SLOT + c * (NTHR * 16), (uint32_t)tid * 16,
                        dst + c * (NTHR * 16));
    };
#pragma unroll
    for (int q = 0; q < kLsRing - 1; ++q) stage(q);
    for (int idx = tid; idx < NETS * NCH * 32; idx += NTHR) c1s[idx] = C1[(size_t)set * NETS * NCH * 32 + idx];
    for (int idx = tid; idx < NETS * 2 * R; idx += NTHR) { // s2, c2: sum of the per-chunk parts
        const int net = idx / (2 * R), rest = idx % (2 * R);
        const float *src = LVp + ((size_t)set * NETS + net) * NCH * 2 * R + rest;
        float acc = 0.f;
        for (int ch = 0; ch < NCH; ++ch) acc += src[(size_t)ch * 2 * R];
        lv[idx] = acc;
    }

    // B operands of the first layer: the rows of X, normalised (zero mean, unit variance)
    op8 xfr[TT][KS];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const size_t row = row0 + wave * (32 * TT) + 32 * tt + x;
        float xv[KS][8];
        float sum = 0.f, sq = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const bf16x8 raw = *(const bf16x8 *)&X[row * D + 16 * s + 8 * h];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                xv[s][e] = (float)raw[e];
                sum += xv[s][e];
                sq += xv[s][e] * xv[s][e];
            }
        }
        sum += __shfl_xor(sum, 32);
        sq += __shfl_xor(sq, 32);
        const float mean = sum * (1.0f / D), var = sq * (1.0f / D) - mean * mean;
        const float inv = rsqrtf(fmaxf(var, 0.f) + 1e-6f);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) xfr[tt][s][e] = (typename Op::elem)((xv[s][e] - mean) * inv);
    }

    // a node's sketch (accumulator registers, lane = token) -> normalised B operands of the
    // network that takes it as input; steps past R / 16 are zero (so are their weights)
    auto normalised = [&](const f32x16 (&mv)[TT][OT], op8 (&dst)[TT][KS]) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            float sum = 0.f, sq = 0.f;
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    sum += mv[tt][ot][v];
                    sq += mv[tt][ot][v] * mv[tt][ot][v];
                }
            sum += __shfl_xor(sum, 32);
            sq += __shfl_xor(sq, 32);
            const float mean = sum * (1.0f / R), var = sq * (1.0f / R) - mean * mean;
            const float inv = rsqrtf(fmaxf(var, 0.f) + 1e-6f);
#pragma unroll
            for (int t = 0; t < KS; ++t) {
                if (t < RS) {
                    f32x8 nv;
#pragma unroll
                    for (int e = 0; e < 8; ++e) nv[e] = (mv[tt][t / 2][8 * (t % 2) + e] - mean) * inv;
                    dst[tt][t] = Op::cvt(nv);
                } else {
                    dst[tt][t] = op8{0};
                }
            }
        }
    };
    static_assert(RS <= KS, "a sketch is no wider than a row");

    f32x16 f1[TT][OT];
    f32x16 node_a[P_DEG == 8 ? TT : 1][P_DEG == 8 ? OT : 1];   // degree 8: the first node's sketch
    op8 xin_b[P_DEG == 8 ? TT : 1][KS];                     // degree 8: input of network 5
    int q = 0;
#pragma unroll 1
    for (int net = 0; net < NETS; ++net) {
        // ---- layers 1 and 2: P2 = gelu(LN(x) W1) (g2 . W2), with the sums for the second LN ----
        f32x16 acc2[TT][OT];
        float sh[TT], sqh[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            sh[tt] = sqh[tt] = 0.f;
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) acc2[tt][ot] = f32x16{0};
        }
#pragma unroll 1
        for (int ch = 0; ch < NCH; ++ch, ++q) {
            wait_vmem_le<(kLsRing - 2) * DMA>();
            __syncthreads();                               // slot q has landed for everybody; slot q-1 is free
            stage(q + kLsRing - 1);
            const unsigned char *sl = ring + (q % kLsRing) * SLOT;
            op8 a1[KS], a2[OT][2];
#pragma unroll
            for (int s = 0; s < KS; ++s) a1[s] = *(const op8 *)(sl + ((s * 32 + x) * 2 + h) * 16);
            f32x16 init;                                   // b1 W1 of this chunk's hidden rows
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 c = *(const f32x4 *)&c1s[(net * NCH + ch) * 32 + 8 * g4 + 4 * h];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) init[4 * g4 + j2] = c[j2];
            }
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    a2[ot][s] = *(const op8 *)(sl + PART1 + (((ot * 2 + s) * 32 + x) * 2 + h) * 16);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                f32x16 acc = init;
#pragma unroll
                for (int s = 0; s < KS; ++s) acc = Op::mfma(a1[s], xfr[tt][s], acc);   // (xfr: this network's input)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float hv = gelu_poly(acc[v]);
                    sh[tt] += hv;
                    sqh[tt] += hv * hv;
                    acc[v] = hv;
                }
                const op8 hf0 = ls_cvt_from16<Op>(acc, 0), hf1 = ls_cvt_from16<Op>(acc, 8);
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) {
                    acc2[tt][ot] = Op::mfma(a2[ot][0], hf0, acc2[tt][ot]);
                    acc2[tt][ot] = Op::mfma(a2[ot][1], hf1, acc2[tt][ot]);
                }
            }
        }
        // ---- second layer normalisation applied to the accumulated product ----
        op8 h2f[TT][RS];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const float s_all = sh[tt] + __shfl_xor(sh[tt], 32), q_all = sqh[tt] + __shfl_xor(sqh[tt], 32);
            const float mean = s_all * (1.0f / HID), var = q_all * (1.0f / HID) - mean * mean;
            const float inv = rsqrtf(fmaxf(var, 0.f) + 1e-6f);
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f32x4 s2 = *(const f32x4 *)&lv[(net * 2 + 0) * R + 32 * ot + 8 * g4 + 4 * h];
                    const f32x4 c2 = *(const f32x4 *)&lv[(net * 2 + 1) * R + 32 * ot + 8 * g4 + 4 * h];
#pragma unroll
                    for (int j2 = 0; j2 < 4; ++j2)
                        acc2[tt][ot][4 * g4 + j2] = (acc2[tt][ot][4 * g4 + j2] - mean * s2[j2]) * inv + c2[j2];
                }
                h2f[tt][2 * ot] = ls_cvt_from16<Op>(acc2[tt][ot], 0);
                h2f[tt][2 * ot + 1] = ls_cvt_from16<Op>(acc2[tt][ot], 8);
            }
        }
        // ---- layers 3 and 4: out = gelu(h2 W3) W4 ----
        f32x16 out[TT][OT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) out[tt][ot] = f32x16{0};
#pragma unroll 1
        for (int ch = 0; ch < NCH; ++ch, ++q) {
            wait_vmem_le<(kLsRing - 2) * DMA>();
            __syncthreads();
            stage(q + kLsRing - 1);
            const unsigned char *sl = ring + (q % kLsRing) * SLOT;
            op8 a3[RS], a4[OT][2];
#pragma unroll
            for (int t = 0; t < RS; ++t) a3[t] = *(const op8 *)(sl + ((t * 32 + x) * 2 + h) * 16);
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    a4[ot][s] = *(const op8 *)(sl + PART1 + (((ot * 2 + s) * 32 + x) * 2 + h) * 16);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                f32x16 acc = {0};
#pragma unroll
                for (int t = 0; t < RS; ++t) acc = Op::mfma(a3[t], h2f[tt][t], acc);
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = gelu_poly(acc[v]);
                const op8 hf0 = ls_cvt_from16<Op>(acc, 0), hf1 = ls_cvt_from16<Op>(acc, 8);
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) {
                    if (QSIDE || net < NETS - 2) {         // [feature][token]
                        out[tt][ot] = Op::mfma(a4[ot][0], hf0, out[tt][ot]);
                        out[tt][ot] = Op::mfma(a4[ot][1], hf1, out[tt][ot]);
                    } else {                               // [token][feature]: lanes = sketch columns
                        out[tt][ot] = Op::mfma(hf0, a4[ot][0], out[tt][ot]);
                        out[tt][ot] = Op::mfma(hf1, a4[ot][1], out[tt][ot]);
                    }
                }
            }
        }
        if ((net & 1) == 0) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) f1[tt][ot] = out[tt][ot];
        } else {
            const float sr = sqrtf((float)R), isr = 1.0f / sr;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                    for (int v = 0; v < 16; ++v) f1[tt][ot][v] = sr * tanh_fast(f1[tt][ot][v] * out[tt][ot][v] * isr);
        }
        if constexpr (P_DEG == 8) {
            if (net == 1) {                                // first node done: keep it, x is still the input
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int ot = 0; ot < OT; ++ot) node_a[tt][ot] = f1[tt][ot];
            } else if (net == 3) {                         // both nodes: they are the inputs from here on
                normalised(f1, xin_b);
                normalised(node_a, xfr);
            } else if (net == 4) {
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int s = 0; s < KS; ++s) xfr[tt][s] = xin_b[tt][s];
            }
        }
    }
    wait_vmem_le<0>();                                     // drain the clamped copies

    // ---- f1 now holds m ----
    if (QSIDE) {
        // lane = token x, register v = sketch column 32 ot + 8 (v / 4) + 4 h + v % 4
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const size_t row = row0 + wave * (32 * TT) + 32 * tt + x;
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f32x4 m4 = {f1[tt][ot][4 * g4], f1[tt][ot][4 * g4 + 1], f1[tt][ot][4 * g4 + 2],
                                      f1[tt][ot][4 * g4 + 3]};
                    *(bf16x4 *)&M_rm[row * R + 32 * ot + 8 * g4 + 4 * h] = cvt4(m4);
                }
        }
    } else {
        // lane = sketch column 32 ot + x, register v = token 8 (v / 4) + 4 h + v % 4 of the tile
        f32x16 sacc[OT][OT];
#pragma unroll
        for (int i = 0; i < OT; ++i)
#pragma unroll
            for (int j2 = 0; j2 < OT; ++j2) sacc[i][j2] = f32x16{0};
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const size_t tile0 = row0 + wave * (32 * TT) + 32 * tt;
#pragma unroll
            for (int ot = 0; ot < OT; ++ot)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f32x4 m4 = {f1[tt][ot][4 * g4], f1[tt][ot][4 * g4 + 1], f1[tt][ot][4 * g4 + 2],
                                      f1[tt][ot][4 * g4 + 3]};
                    const size_t oct = (tile0 >> 3) + g4;
                    *(f32x4 *)&M8[((oct * 2 + h) * R + 32 * ot + x) * 4] = m4;
                }
            // S += m^T m over the tile: the registers, eight at a time, are A and B fragments at
            // once (k = token, same order on both sides)
#pragma unroll
            for (int sp = 0; sp < 2; ++sp) {
                bf16x8 f[OT];
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) f[ot] = cvt8_from16(f1[tt][ot], 8 * sp);
#pragma unroll
                for (int i = 0; i < OT; ++i)
#pragma unroll
                    for (int j2 = 0; j2 < OT; ++j2) sacc[i][j2] = mfma32(f[i], f[j2], sacc[i][j2]);
            }
        }
        float *outp = Spart + (size_t)blockIdx.x * R * R;
        float *red = (float *)ring;                        // [NW][32][32]; the ring is idle by now
#pragma unroll
        for (int i = 0; i < OT; ++i)
#pragma unroll
            for (int j2 = 0; j2 < OT; ++j2) {
                __syncthreads();
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    red[(wave * 32 + 8 * (v / 4) + 4 * h + (v % 4)) * 32 + x] = sacc[i][j2][v];
                __syncthreads();
                for (int idx = tid; idx < 32 * 32; idx += NTHR) {
                    float sum = 0.f;
#pragma unroll
                    for (int wv = 0; wv < NW; ++wv) sum += red[wv * 1024 + idx];
                    outp[(size_t)(32 * i + idx / 32) * R + 32 * j2 + idx % 32] = sum;
                }
            }
    }
}

int sketch_tiles_per_wg(int b);

struct MfmaWs {
    bf16_t *Gt; bf16_t *MQ; float *MK8; bf16_t *V8; bf16_t *Zg; float *Spart; bf16_t *Shi, *Slo;
    float *Pnum, *Pden;                          // in-block part of the rows (two-launch output, see k_out)
    _Float16 *V8h; float *Kscale;                // half-precision state kernel: value octets, key scales per part
    float *M32;                                  // learned sketches only: m(x) as fp32 rows
    bf16_t *MKrm;                                // m(K) as bf16 rows: in-block rule of Section 3.1 only
    bf16_t *LW; float *C1, *LVp;                 // learned sketches on MFMA: arranged weights
    size_t total;
};

// Learned sketches of degree 4 and 8 with d = 64 or 128 run on MFMA when a 256-token workgroup stays
// inside one block; everything else goes through the general fp32 sketch kernel.
bool learned_on_mfma(const Problem &pb)
{
    return pb.learned && (pb.p == 4 || pb.p == 8) && (pb.d == 64 || pb.d == 128) && pb.b % 256 == 0;
}

// tokens per partial S = m^T m handed to the denominator scan
int part_tokens(const Problem &pb) { return learned_on_mfma(pb) ? 256 : 128 * sketch_tiles_per_wg(pb.b); }

int sketch_tiles_per_wg(int b)
{
    int tiles = 8;                               // workgroup = 128 * tiles tokens, inside one block
    while (b % (tiles * 128) != 0) tiles /= 2;
    return tiles;
}

// The causal call with exact in-block weights at d = r = 64 runs the in-block part of the output
// beside the state kernel when the state kernel leaves room for it: at most one state
// workgroup per CU (ten per unit) and at least one prefix state to compute.
constexpr int kComputeUnits = 256;
// From this many rows per tensor on, the sketches and layouts are HBM-bound whatever the number
// of launches, and the separate kernels (matrices transposed once, straight copies into LDS)
// move the bytes 5 to 13 % faster than k_prep's roles; below, fewer launches win.
constexpr size_t kPrepMaxRows = (size_t)1 << 22;
bool in_block_beside_states(const Problem &pb)
{
    // (and at most 512 tiles of 128 tokens per unit: the half-precision state kernel keeps their scales in LDS)
    return pb.d == 64 && pb.r == 64 && pb.local_exact && pb.t >= 2 && pb.units * 10 <= kComputeUnits &&
           pb.n / 128 <= 512;
}

// The causal call with Gaussian sketches of degree 4, exact in-block weights and r = d = 64 forms its
// prefix states from fp16 products (fp16 key sketches with a scale per 128-token tile, fp16 values),
// beside the in-block part where that applies, else as a launch of its own.
bool half_precision_states(const Problem &pb)
{
    // (either in-block rule: with Section 3.1's the key role also leaves the bf16 rows of m(K))
    return pb.d == 64 && pb.r == 64 && pb.p == 4 && !pb.learned && pb.t >= 2 && pb.b % 256 == 0 &&
           pb.n / 128 <= kStateF16Tiles;
}

MfmaWs carve(const Problem &pb, void *ws)
{
    MfmaWs w;
    const size_t rows = (size_t)pb.units * pb.n, R = pb.r, D = pb.d, tb = pb.t > 1 ? pb.t - 1 : 0;
    const size_t sets = pb.per_head ? pb.heads : 1;
    const size_t parts = rows / (size_t)part_tokens(pb);
    size_t off = 0;
    char *base = (char *)ws;
    auto take = [&](size_t bytes) { char *p = base + off; off += align_up(bytes, 256); return p; };
    w.Gt = (bf16_t *)take(pb.learned ? 0 : sets * pb.g_len * 2);
    w.MQ = (bf16_t *)take(pb.p == 2 ? 0 : rows * R * 2);     // p = 2: m(Q) = Q itself
    w.MK8 = (float *)take(rows * R * 4);
    w.V8 = (bf16_t *)take(rows * D * 2);
    w.Zg = (bf16_t *)take((size_t)pb.units * tb * R * R * D * 2);
    w.Spart = (float *)take(parts * R * R * 4);
    w.Shi = (bf16_t *)take((size_t)pb.units * tb * R * R * 2);
    w.Slo = (bf16_t *)take((size_t)pb.units * tb * R * R * 2);
    w.MKrm = (bf16_t *)take(pb.local_exact ? 0 : rows * R * 2);
    w.Pnum = (float *)take(in_block_beside_states(pb) ? rows * D * 4 : 0);
    w.Pden = (float *)take(in_block_beside_states(pb) ? rows * 2 * 4 : 0);
    w.V8h = (_Float16 *)take(half_precision_states(pb) ? rows * D * 2 : 0);
    w.Kscale = (float *)take(half_precision_states(pb) ? rows / 128 * 4 : 0);
    const bool fast_learned = learned_on_mfma(pb);
    w.M32 = (float *)take(pb.learned && !fast_learned ? rows * R * 4 : 0);
    const size_t nch = R / 4;                            // hidden chunks of 32 (8 R wide)
    const size_t nets = pb.p > 2 ? pb.p - 2 : 0;         // networks per set
    w.LW = (bf16_t *)take(fast_learned ? sets * 2 * nets * nch * ls_slot_bytes(pb.d) : 0);
    w.C1 = (float *)take(fast_learned ? sets * nets * nch * 32 * 4 : 0);
    w.LVp = (float *)take(fast_learned ? sets * nets * nch * 2 * R * 4 : 0);
    w.total = off;
    return w;
}

psf_status launch_transpose_g(const Problem &pb, const void *G, bf16_t *Gt, hipStream_t s)
{
    const int nmat = pb.p / 2 + (pb.p / 2 >= 4 ? pb.p / 2 - 2 : 0);
    hipLaunchKernelGGL(k_transpose_g, dim3(nmat, pb.per_head ? pb.heads : 1), dim3(kWg), 0, s,
                       (const bf16_t *)G, Gt, pb.d, pb.r, pb.p, pb.g_len);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}

template <int D, int R, int P>
psf_status launch_sketch(const Problem &pb, const void *X, const bf16_t *Gt, bool qside, bf16_t *M_rm,
                         float *M8, float *Spart, int tiles, hipStream_t s)
{
    const unsigned grid = (unsigned)((size_t)pb.units * pb.n / (128 * (size_t)tiles));
    if (qside)
        hipLaunchKernelGGL((k_sketch<D, R, P, true>), dim3(grid), dim3(kWg), 0, s, (const bf16_t *)X, Gt,
                           pb.n, pb.heads, pb.per_head ? 1 : 0, pb.g_len, tiles, M_rm, M8, Spart);
    else
        hipLaunchKernelGGL((k_sketch<D, R, P, false>), dim3(grid), dim3(kWg), 0, s, (const bf16_t *)X, Gt,
                           pb.n, pb.heads, pb.per_head ? 1 : 0, pb.g_len, tiles, M_rm, M8, Spart);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}

// The symmetric deal of the state kernel at d = 128, r = 64: ten workgroups per unit instead of
// sixteen with the same work each (config 5: 0.285 -> 0.254 ms for the state stage).
constexpr bool kSymWide = true;
// Running prefix states of (M8, V8) for every unit, snapshots into Zg.
template <int D, int R>
psf_status launch_state(const Problem &pb, const float *M8, const bf16_t *V8, bf16_t *Zg, hipStream_t s)
{
    // Symmetric deal (d = 64): only the (a, 16-wide column range) segments the output kernel
    // reads.  For r = 32 it pays once the grid is a few workgroups per CU; small grids keep
    // the full tiles with four per wave, which fill the CUs better.
    constexpr int GROUPS = (R / 16) * (R / 16 + 1) / 2;
    const unsigned grid_sym = (unsigned)(pb.units * GROUPS);
    if (D == 64 && (R == 64 || grid_sym > 512)) {
        if constexpr (D == 64) {
            // One block only (no mask, or the prompt of a decode): eight waves, two per SIMD,
            // 8 % faster per token; with a snapshot every block the exchange and the stalled
            // ring after the stores cost more than that.
            // (r = 32 reaches this branch with large grids only.)
            if (R == 64 && grid_sym <= 256 && pb.t == 2) {
                if constexpr (R == 64)
                    hipLaunchKernelGGL((k_state_two_waves<R, D, 64>), dim3(grid_sym), dim3(2 * kWg), 0, s, M8, V8,
                                       Zg, pb.n, pb.b, pb.t, pb.units);
            } else if (grid_sym <= 256)
                hipLaunchKernelGGL((k_state<R, D, 2, true, 64, 1>), dim3(grid_sym), dim3(kWg), 0, s, M8, V8, Zg,
                                   pb.n, pb.b, pb.t, pb.units);
            else
                hipLaunchKernelGGL((k_state<R, D, 2, true, 32, 2>), dim3(grid_sym), dim3(kWg), 0, s, M8, V8, Zg,
                                   pb.n, pb.b, pb.t, pb.units);
        }
    } else if (D == 128 && R == 64 && kSymWide) {
        if constexpr (D == 128 && R == 64)
            hipLaunchKernelGGL((k_state<R, D, 2, true, 64, 1>), dim3(grid_sym), dim3(kWg), 0, s, M8, V8, Zg, pb.n, pb.b,
                               pb.t, pb.units);
    } else if constexpr (!(D == 64 && R == 64)) {
        constexpr int NA = (D == 64) ? 4 : 2;
        constexpr int AG = NA * 4 / (R / 32);
        const unsigned grid = (unsigned)(pb.units * (R / AG));
        hipLaunchKernelGGL((k_state<R, D, NA, false, 64, 1>), dim3(grid), dim3(kWg), 0, s, M8, V8, Zg, pb.n,
                           pb.b, pb.t, pb.units);
    }
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}

// Den (1 + sum of weights per row, fp32) and MK_rm (m(K) as bf16 rows) are extra outputs the
// backward pass asks for; the forward entry point passes null.
template <int D, int R, int P>
psf_status attn_impl(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                     void *O, void *ws, hipStream_t s, StageTimer *tm, float *Den = nullptr,
                     bf16_t *MK_rm = nullptr, bool noncausal = false)
{
    MfmaWs w = carve(pb, ws);
    const int tiles = sketch_tiles_per_wg(pb.b);
    psf_status st;
    bool v_done = false;                         // value octets already written by the sketch launch
    // the state kernel's launch also runs the in-block part of the output, the denominator scan
    // and, with Gaussian sketches of degree 4, the sketch of the query rows
    // (the backward pass's forward, which also wants the denominators: Gaussian sketches of degree 4 only)
    const bool beside = D == 64 && R == 64 && P != 2 && in_block_beside_states(pb) && !noncausal &&
                        (!Den || (P == 4 && !pb.learned));
    const bool q_beside = beside && P == 4 && !pb.learned;
    // the same state kernel without the fused launch (more state workgroups than CUs)
    const bool f16_alone = D == 64 && R == 64 && P == 4 && half_precision_states(pb) && !beside && !noncausal && !Den &&
                           !MK_rm;
    if (pb.learned) {
        const size_t rows = (size_t)pb.units * pb.n, count = rows * R;
        bool fast = false;
        if constexpr (P == 4 || P == 8) {
            if (learned_on_mfma(pb)) {
                fast = true;
                const int sets = pb.per_head ? pb.heads : 1;
                const unsigned grid = (unsigned)(rows / 256);
                hipLaunchKernelGGL((k_learned_prep<R, P, D>), dim3(2 * (P - 2) * (R / 4), sets), dim3(kWg), 0, s,
                                   (const bf16_t *)G, pb.g_len, w.LW, w.C1, w.LVp);
                PSF_LAUNCH_CHECK();
                constexpr int TT = 1;                       // 8 waves of one tile: two waves per SIMD
                hipLaunchKernelGGL((k_learned_sketch<R, true, TT, P, D>), dim3(grid), dim3(512 / TT), 0, s,
                                   (const bf16_t *)Q, w.LW, w.C1, w.LVp, w.MQ, nullptr, nullptr, pb.n, pb.heads,
                                   pb.per_head ? 1 : 0);
                PSF_LAUNCH_CHECK();
                hipLaunchKernelGGL((k_learned_sketch<R, false, TT, P, D>), dim3(grid), dim3(512 / TT), 0, s,
                                   (const bf16_t *)K, w.LW, w.C1, w.LVp, nullptr, w.MK8, w.Spart, pb.n, pb.heads,
                                   pb.per_head ? 1 : 0);
                PSF_LAUNCH_CHECK();
            }
        }
        if (!fast) {
            // other degrees and shapes: the general fp32 sketch kernel, then the layouts
            st = general_sketch_f32(pb, Q, G, w.M32, s);
            if (st != PSF_OK) return st;
            hipLaunchKernelGGL(k_m_to_bf16, dim3((unsigned)((count / 4 + kWg - 1) / kWg)), dim3(kWg), 0, s,
                               w.M32, w.MQ, count);
            PSF_LAUNCH_CHECK();
            st = general_sketch_f32(pb, K, G, w.M32, s);
            if (st != PSF_OK) return st;
            hipLaunchKernelGGL((k_m_to_octets_and_partials<R>), dim3((unsigned)(rows / part_tokens(pb))),
                               dim3(kWg), 0, s, w.M32, w.MK8, w.Spart, part_tokens(pb));
            PSF_LAUNCH_CHECK();
        }
    } else if constexpr (P == 2) {
        // base case of Algorithm 1: m(x) = x (r = d).  The query rows serve as m(Q) as they are;
        // the key rows are put into the state kernel's layout (and their m^T m partials formed).
        static_assert(R == D, "p = 2: the sketch is the row itself");
        const size_t rows = (size_t)pb.units * pb.n;
        w.MQ = (bf16_t *)Q;
        hipLaunchKernelGGL((k_m_to_octets_and_partials<R, bf16_t>), dim3((unsigned)(rows / part_tokens(pb))),
                           dim3(kWg), 0, s, (const bf16_t *)K, w.MK8, w.Spart, part_tokens(pb));
        PSF_LAUNCH_CHECK();
    } else if (P == 4 && (q_beside || f16_alone || (size_t)pb.units * pb.n < kPrepMaxRows)) {
      if constexpr (P == 4) {
        // degree 4 with Gaussian sketches: query sketch + value layout in one launch, key sketch
        const unsigned parts = (unsigned)((size_t)pb.units * pb.n / (128 * (size_t)tiles));
        if (Den || MK_rm) {                      // the backward pass reads the transposed matrices
            st = launch_transpose_g(pb, G, w.Gt, s);
            if (st != PSF_OK) return st;
        }
        bf16_t *mk_rows = MK_rm ? MK_rm : (pb.local_exact ? nullptr : w.MKrm);
        if (f16_alone) {
            hipLaunchKernelGGL((k_prep<D, R, false, true>), dim3(2 * parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                               (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                               pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 1, w.Kscale,
                               w.V8h);
            PSF_LAUNCH_CHECK();
            if (mk_rows)
                hipLaunchKernelGGL((k_prep<D, R, true, true, true>), dim3(parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                                   (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                                   pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 1,
                                   w.Kscale, w.V8h);
            else
                hipLaunchKernelGGL((k_prep<D, R, true, true>), dim3(parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                                   (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                                   pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 1,
                                   w.Kscale, w.V8h);
            PSF_LAUNCH_CHECK();
        } else if (q_beside) {
            // the state kernel of this path works in half precision: fp16 value octets and key sketches
            hipLaunchKernelGGL((k_prep<D, R, false, true>), dim3(parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                               (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                               pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 0, w.Kscale,
                               w.V8h);
            PSF_LAUNCH_CHECK();
            if (mk_rows)
                hipLaunchKernelGGL((k_prep<D, R, true, true, true>), dim3(parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                                   (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                                   pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 1,
                                   w.Kscale, w.V8h);
            else
                hipLaunchKernelGGL((k_prep<D, R, true, true>), dim3(parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                                   (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                                   pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 1,
                                   w.Kscale, w.V8h);
            PSF_LAUNCH_CHECK();
        } else {
            hipLaunchKernelGGL((k_prep<D, R, false>), dim3(2 * parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                               (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                               pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 1, nullptr,
                               nullptr);
            PSF_LAUNCH_CHECK();
            hipLaunchKernelGGL((k_prep<D, R, true>), dim3(parts), dim3(kWg), 0, s, (const bf16_t *)Q,
                               (const bf16_t *)K, (const bf16_t *)V, (const bf16_t *)G, pb.n, pb.heads,
                               pb.per_head ? 1 : 0, pb.g_len, tiles, w.MQ, w.MK8, mk_rows, w.Spart, w.V8, 1, nullptr,
                               nullptr);
            PSF_LAUNCH_CHECK();
        }
        v_done = true;
      }
    } else {
        st = launch_transpose_g(pb, G, w.Gt, s);
        if (st != PSF_OK) return st;
        st = launch_sketch<D, R, P>(pb, Q, w.Gt, true, w.MQ, nullptr, nullptr, tiles, s);
        if (st != PSF_OK) return st;
        st = launch_sketch<D, R, P>(pb, K, w.Gt, false, MK_rm ? MK_rm : (pb.local_exact ? nullptr : w.MKrm), w.MK8,
                                    w.Spart, tiles, s);
        if (st != PSF_OK) return st;
    }
    if (!v_done) {
        const size_t octets = (size_t)pb.units * pb.n / 8;
        hipLaunchKernelGGL((k_v_octets<D>), dim3((unsigned)((octets * D + kWg - 1) / kWg)), dim3(kWg), 0,
                           s, (const bf16_t *)V, w.V8, octets);
        PSF_LAUNCH_CHECK();
    }
    if (tm) tm->mark();
    if (pb.t > 1 && !beside) {
        hipLaunchKernelGGL((k_den_scan<R>), dim3(R * R / kWg, pb.units), dim3(kWg), 0, s, w.Spart, w.Shi,
                           w.Slo, pb.t, pb.b / part_tokens(pb), pb.n / part_tokens(pb));
        PSF_LAUNCH_CHECK();
    }
    if (tm) tm->mark();
    if constexpr (D == 64 && R == 64 && P != 2) {
        if (beside) {
            constexpr int TT = 2;
            const int n_tiles = pb.units * (pb.n / (128 * TT));
            const int n_q = q_beside ? (int)((size_t)pb.units * pb.n / (128 * (size_t)tiles)) : 0;
            BesideStates a;
            a.Q = (const bf16_t *)Q; a.K = (const bf16_t *)K; a.G = (const bf16_t *)G;
            a.Pnum = w.Pnum; a.Pden = w.Pden; a.MQ = w.MQ;
            a.Spart = w.Spart; a.Shi = w.Shi; a.Slo = w.Slo;
            a.heads = pb.heads; a.per_head = pb.per_head ? 1 : 0; a.tiles_per_wg = tiles;
            a.parts_per_block = pb.b / part_tokens(pb); a.parts_per_unit = pb.n / part_tokens(pb);
            a.n_state = pb.units * 10; a.n_den = pb.units * (R * R / kWg);
            a.n_tiles = n_tiles;
            a.ratio = n_q > 0 ? n_tiles / n_q : n_tiles;       // tiles between two sketch parts (exact: both tile n)
            a.g_len = pb.g_len;
            a.V8h = w.V8h; a.Kscale = w.Kscale;
            const dim3 grid((unsigned)(a.n_state + a.n_den + n_tiles + n_q));
            if (q_beside)
                hipLaunchKernelGGL((k_state_and_in_block<R, D, P, TT, true>), grid, dim3(kWg), 0, s, w.MK8, w.V8, w.Zg,
                                   pb.units, pb.n, pb.b, pb.t, a);
            else
                hipLaunchKernelGGL((k_state_and_in_block<R, D, P, TT, false>), grid, dim3(kWg), 0, s, w.MK8, w.V8, w.Zg,
                                   pb.units, pb.n, pb.b, pb.t, a);
            PSF_LAUNCH_CHECK();
            if (tm) tm->mark();
            if (Den)
                hipLaunchKernelGGL((k_out<R, D, P, TT, true, false, false, 2>), dim3((unsigned)n_tiles), dim3(kWg), 0, s,
                                   (const bf16_t *)Q, (const bf16_t *)K, w.V8, w.MQ, w.Zg, w.Shi, w.Slo, (bf16_t *)O,
                                   Den, w.Pnum, w.Pden, pb.n, pb.b, pb.t);
            else
                hipLaunchKernelGGL((k_out<R, D, P, TT, false, false, false, 2>), dim3((unsigned)n_tiles), dim3(kWg), 0, s,
                                   (const bf16_t *)Q, (const bf16_t *)K, w.V8, w.MQ, w.Zg, w.Shi, w.Slo, (bf16_t *)O,
                                   nullptr, w.Pnum, w.Pden, pb.n, pb.b, pb.t);
            PSF_LAUNCH_CHECK();
            if (tm) tm->mark();
            return PSF_OK;
        }
    }
    if (f16_alone) {
        if constexpr (D == 64 && R == 64) {
            hipLaunchKernelGGL((k_state_f16<R, D>), dim3((unsigned)(pb.units * 10)), dim3(kWg), 0, s,
                               (const _Float16 *)w.MK8, w.V8h, w.Kscale, w.Zg, pb.n, pb.b, pb.t, pb.units);
            PSF_LAUNCH_CHECK();
        }
    } else if (pb.t > 1) {
        st = launch_state<D, R>(pb, w.MK8, w.V8, w.Zg, s);
        if (st != PSF_OK) return st;
    }
    if (tm) tm->mark();
    {
        // tokens per workgroup = 128 * TT.  (TT = 4 halves the LDS traffic per token but needs
        // one workgroup per CU; it measured 1.7x slower than TT = 2 with two per CU.)
        constexpr int TT = (D == 64) ? 2 : 1;
        const unsigned grid = (unsigned)((size_t)pb.units * (pb.n / (128 * TT)));
        constexpr bool LS_OK = (32 * TT * R * 2) % (16 * kWg) == 0;    // whole copies of a key tile of m(K) rows
        if (!noncausal && !pb.local_exact) {
            if constexpr (LS_OK) {
                if (pb.learned) return PSF_ERR_UNSUPPORTED;         // (not routed here: see select_path)
                const bf16_t *mk_rows = MK_rm ? MK_rm : w.MKrm;
                if (Den) {
                    // the backward pass's forward: only where the backward kernels exist
                    if constexpr (D == 64 && R == 64 && P == 4)
                        hipLaunchKernelGGL((k_out<R, D, P, TT, true, false, true>), dim3(grid), dim3(kWg), 0, s, w.MQ,
                                           mk_rows, w.V8, w.MQ, w.Zg, w.Shi, w.Slo, (bf16_t *)O, Den, nullptr, nullptr, pb.n, pb.b, pb.t);
                    else
                        return PSF_ERR_UNSUPPORTED;
                } else {
                    hipLaunchKernelGGL((k_out<R, D, P, TT, false, false, true>), dim3(grid), dim3(kWg), 0, s, w.MQ,
                                       mk_rows, w.V8, w.MQ, w.Zg, w.Shi, w.Slo, (bf16_t *)O, Den, nullptr, nullptr, pb.n, pb.b, pb.t);
                }
            } else {
                return PSF_ERR_UNSUPPORTED;
            }
        } else if (noncausal)
            hipLaunchKernelGGL((k_out<R, D, P, TT, false, true>), dim3(grid), dim3(kWg), 0, s, (const bf16_t *)Q,
                               (const bf16_t *)K, w.V8, w.MQ, w.Zg, w.Shi, w.Slo, (bf16_t *)O, Den, nullptr, nullptr, pb.n,
                               pb.b, pb.t);
        else if (Den)
            hipLaunchKernelGGL((k_out<R, D, P, TT, true>), dim3(grid), dim3(kWg), 0, s, (const bf16_t *)Q,
                               (const bf16_t *)K, w.V8, w.MQ, w.Zg, w.Shi, w.Slo, (bf16_t *)O, Den, nullptr, nullptr, pb.n,
                               pb.b, pb.t);
        else
            hipLaunchKernelGGL((k_out<R, D, P, TT, false>), dim3(grid), dim3(kWg), 0, s, (const bf16_t *)Q,
                               (const bf16_t *)K, w.V8, w.MQ, w.Zg, w.Shi, w.Slo, (bf16_t *)O, Den, nullptr, nullptr, pb.n,
                               pb.b, pb.t);
        PSF_LAUNCH_CHECK();
    }
    if (tm) tm->mark();
    return PSF_OK;
}

#include "psf_mfma_learned_bwd.inl"
#include "psf_mfma_bwd.inl"

}  // namespace

// p = 2: m(x) = x, so the sketch size is d whatever the descriptor says, and the two in-block
// rules coincide (<m(q), m(k)>^2 = <q, k>^2).
static Problem base_case_problem(const Problem &pb0)
{
    Problem pb = pb0;
    if (pb.p == 2) {
        pb.r = pb.mcols;
        pb.local_exact = true;
    }
    return pb;
}

size_t mfma_workspace_bytes(const Problem &pb) { return carve(base_case_problem(pb), nullptr).total; }

// What the forward call runs inside the state kernel's launch (see k_state_and_in_block):
// bit 0: the in-block part of the output and the denominator scan; bit 1: the query sketch.
int mfma_beside_states(const Problem &pb0)
{
    const Problem pb = base_case_problem(pb0);
    if (!(pb.d == 64 && pb.r == 64 && pb.p != 2 && in_block_beside_states(pb))) return 0;
    return 1 | (pb.p == 4 && !pb.learned ? 2 : 0);
}

bool mfma_bwd_supported(const Problem &pb)
{
    // in-block weights from the sketches (Section 3.1): d = r = 64, degree 4 only;
    // learned sketches (the networks' reverse pass on MFMA): d = 64, degree 4, exact in-block weights
    const bool base = pb.d == 64 && pb.p == 4;
    return (pb.d == 64 || pb.d == 128) && pb.dv == pb.d && (pb.p == 4 || pb.p == 8) && (pb.r == 32 || pb.r == 64) &&
           pb.b % 256 == 0 && !pb.exact_feat && (!pb.learned || base) &&
           (pb.local_exact || (base && pb.r == 64 && !pb.learned));
}

size_t mfma_bwd_workspace_bytes(const Problem &pb) { return carve_bwd(pb, nullptr).total; }

#define PSF_BWD_DISPATCH(CALL)                                               \
    do {                                                                     \
        if (pb.d == 64 && pb.r == 64 && pb.p == 4) return CALL(64, 64, 4);   \
        if (pb.d == 64 && pb.r == 32 && pb.p == 4) return CALL(64, 32, 4);   \
        if (pb.d == 64 && pb.r == 64 && pb.p == 8) return CALL(64, 64, 8);   \
        if (pb.d == 64 && pb.r == 32 && pb.p == 8) return CALL(64, 32, 8);   \
        if (pb.d == 128 && pb.r == 64 && pb.p == 4) return CALL(128, 64, 4); \
        if (pb.d == 128 && pb.r == 32 && pb.p == 4) return CALL(128, 32, 4); \
        if (pb.d == 128 && pb.r == 64 && pb.p == 8) return CALL(128, 64, 8); \
        if (pb.d == 128 && pb.r == 32 && pb.p == 8) return CALL(128, 32, 8); \
        return PSF_ERR_UNSUPPORTED;                                          \
    } while (0)

psf_status mfma_attn_bwd(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                         const void *dO, void *dQ, void *dK, void *dV, void *ws, hipStream_t s, StageTimer *tm,
                         void *saved, const void *O_saved, float *dG)
{
    if (dG && !pb.learned) return PSF_ERR_UNSUPPORTED;
#define PSF_AT(D_, R_, P_) (attn_bwd_impl<R_, D_, P_>(pb, Q, K, V, G, dO, dQ, dK, dV, ws, s, tm, saved, O_saved, dG))
    PSF_BWD_DISPATCH(PSF_AT);
#undef PSF_AT
}

size_t mfma_fwd_save_bytes(const Problem &pb) { return carve_saved(pb, nullptr).total; }

namespace {
template <int D, int R, int P>
psf_status fwd_save_impl(const Problem &pb, const void *Q, const void *K, const void *V, const void *G, void *O,
                         const MfmaSaved &sv, hipStream_t s, StageTimer *tm)
{
    psf_status st = attn_impl<D, R, P>(pb, Q, K, V, G, O, sv.fwd, s, tm, sv.Den, sv.MK);
    if (st != PSF_OK || !pb.learned) return st;
    // (the learned key-side sketch kernel writes the state kernel's octets only)
    if (!learned_on_mfma(pb)) return PSF_ERR_UNSUPPORTED;
    const size_t count4 = (size_t)pb.units * pb.n * R / 4;
    hipLaunchKernelGGL((k_octets_to_rows<R>), dim3((unsigned)((count4 + kWg - 1) / kWg)), dim3(kWg), 0, s,
                       carve(pb, sv.fwd).MK8, sv.MK, count4);
    PSF_LAUNCH_CHECK();
    return PSF_OK;
}
}  // namespace

psf_status mfma_attn_fwd_save(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                              void *O, void *saved, hipStream_t s, StageTimer *tm)
{
    const MfmaSaved sv = carve_saved(pb, saved);
#define PSF_AT(D_, R_, P_) (fwd_save_impl<D_, R_, P_>(pb, Q, K, V, G, O, sv, s, tm))
    PSF_BWD_DISPATCH(PSF_AT);
#undef PSF_AT
}

#define PSF_DISPATCH(CALL)                                                   \
    do {                                                                     \
        if (pb.d == 64 && pb.p == 2) return CALL(64, 64, 2);                 \
        if (pb.d == 64 && pb.r == 64 && pb.p == 4) return CALL(64, 64, 4);   \
        if (pb.d == 64 && pb.r == 32 && pb.p == 4) return CALL(64, 32, 4);   \
        if (pb.d == 64 && pb.r == 64 && pb.p == 8) return CALL(64, 64, 8);   \
        if (pb.d == 64 && pb.r == 32 && pb.p == 8) return CALL(64, 32, 8);   \
        if (pb.d == 128 && pb.r == 64 && pb.p == 4) return CALL(128, 64, 4); \
        if (pb.d == 128 && pb.r == 32 && pb.p == 4) return CALL(128, 32, 4); \
        if (pb.d == 128 && pb.r == 64 && pb.p == 8) return CALL(128, 64, 8); \
        if (pb.d == 128 && pb.r == 32 && pb.p == 8) return CALL(128, 32, 8); \
        return PSF_ERR_UNSUPPORTED;                                          \
    } while (0)

psf_status mfma_attn(const Problem &pb0, const void *Q, const void *K, const void *V, const void *G,
                     void *O, void *ws, hipStream_t s, StageTimer *tm)
{
    const Problem pb = base_case_problem(pb0);
#define PSF_AT(D_, R_, P_) (attn_impl<D_, R_, P_>(pb, Q, K, V, G, O, ws, s, tm))
    PSF_DISPATCH(PSF_AT);
#undef PSF_AT
}

// ---- total state of a run of tokens (for the hand-over from a prompt to token-by-token
// evaluation): Z = sum_j phi'(k_j) v_j^T over the n_tok tokens of every unit, from the sketch,
// layout and state kernels of the forward path run on one "block" of n_tok tokens (as the
// non-causal entry point does).  Zg: [units][a][b'/8][c][8] bf16 with the symmetry weights of
// k_state (b' > a doubled, b' < a zero); Spart: [units][parts][r][r] fp32 partial m^T m.
struct TotalWs {
    bf16_t *Gt; float *MK8; bf16_t *V8; bf16_t *Zg; float *Spart;
    bf16_t *LW; float *C1, *LVp;                 // learned sketches: arranged weights (see k_learned_prep)
    size_t total;
};

static Problem total_problem(const Problem &pb0, int n_tok)
{
    Problem pb = pb0;
    pb.n = n_tok;
    pb.b = n_tok;
    pb.t = 2;
    pb.local_exact = true;
    return pb;
}

static TotalWs carve_total(const Problem &pb, void *ws)
{
    TotalWs w;
    const size_t rows = (size_t)pb.units * pb.n, R = pb.r, D = pb.d;
    const size_t sets = pb.per_head ? pb.heads : 1, parts = rows / (size_t)part_tokens(pb);
    size_t off = 0;
    char *base = (char *)ws;
    auto take = [&](size_t bytes) { char *q = base + off; off += align_up(bytes, 256); return q; };
    w.Gt = (bf16_t *)take(pb.learned ? 0 : sets * pb.g_len * 2);
    w.MK8 = (float *)take(rows * R * 4);
    w.V8 = (bf16_t *)take(rows * D * 2);
    w.Zg = (bf16_t *)take((size_t)pb.units * R * R * D * 2);
    w.Spart = (float *)take(parts * R * R * 4);
    const size_t nch = R / 4;
    w.LW = (bf16_t *)take(pb.learned ? sets * 4 * nch * kLsSlotBytes : 0);
    w.C1 = (float *)take(pb.learned ? sets * 2 * nch * 32 * 4 : 0);
    w.LVp = (float *)take(pb.learned ? sets * 2 * nch * 2 * R * 4 : 0);
    w.total = off;
    return w;
}

bool mfma_total_state_supported(const Problem &pb, int n_tok)
{
    const bool shapes = pb.bf16 && !pb.exact_feat && pb.d == pb.dv && (pb.d == 64 || pb.d == 128) &&
                        (pb.r == 32 || pb.r == 64) && n_tok >= 256 && n_tok % 256 == 0;
    // learned sketches: the MFMA sketch kernel exists for degree 4 and d = 64
    return shapes && (pb.learned ? pb.p == 4 && pb.d == 64 : pb.p == 4 || pb.p == 8);
}

size_t mfma_total_state_workspace_bytes(const Problem &pb, int n_tok)
{
    return carve_total(total_problem(pb, n_tok), nullptr).total;
}

namespace {
template <int D, int R, int P>
psf_status total_state_impl(const Problem &pb, const void *K, const void *V, const void *G, const TotalWs &w,
                            hipStream_t s)
{
    psf_status st;
    if (pb.learned) {
        if constexpr (P == 4 && D == 64) {
            const int sets = pb.per_head ? pb.heads : 1;
            hipLaunchKernelGGL((k_learned_prep<R>), dim3(4 * (R / 4), sets), dim3(kWg), 0, s, (const bf16_t *)G,
                               pb.g_len, w.LW, w.C1, w.LVp);
            PSF_LAUNCH_CHECK();
            hipLaunchKernelGGL((k_learned_sketch<R, false, 1>), dim3((unsigned)((size_t)pb.units * pb.n / 256)),
                               dim3(512), 0, s, (const bf16_t *)K, w.LW, w.C1, w.LVp, nullptr, w.MK8, w.Spart, pb.n,
                               pb.heads, pb.per_head ? 1 : 0);
            PSF_LAUNCH_CHECK();
        } else {
            return PSF_ERR_UNSUPPORTED;
        }
    } else {
        st = launch_transpose_g(pb, G, w.Gt, s);
        if (st != PSF_OK) return st;
        st = launch_sketch<D, R, P>(pb, K, w.Gt, false, nullptr, w.MK8, w.Spart, sketch_tiles_per_wg(pb.b), s);
        if (st != PSF_OK) return st;
    }
    const size_t octets = (size_t)pb.units * pb.n / 8;
    hipLaunchKernelGGL((k_v_octets<D>), dim3((unsigned)((octets * D + kWg - 1) / kWg)), dim3(kWg), 0, s,
                       (const bf16_t *)V, w.V8, octets);
    PSF_LAUNCH_CHECK();
    return launch_state<D, R>(pb, w.MK8, w.V8, w.Zg, s);
}
}  // namespace

psf_status mfma_total_state(const Problem &pb0, int n_tok, const void *K, const void *V, const void *G, void *ws,
                            hipStream_t s, const void **Zg, const float **Spart, int *parts_per_unit)
{
    const Problem pb = total_problem(pb0, n_tok);
    const TotalWs w = carve_total(pb, ws);
    *Zg = w.Zg;
    *Spart = w.Spart;
    *parts_per_unit = pb.n / part_tokens(pb);
#define PSF_AT(D_, R_, P_) (total_state_impl<D_, R_, P_>(pb, K, V, G, w, s))
    if (pb.d == 64 && pb.r == 64 && pb.p == 4) return PSF_AT(64, 64, 4);
    if (pb.d == 64 && pb.r == 32 && pb.p == 4) return PSF_AT(64, 32, 4);
    if (pb.d == 64 && pb.r == 64 && pb.p == 8) return PSF_AT(64, 64, 8);
    if (pb.d == 64 && pb.r == 32 && pb.p == 8) return PSF_AT(64, 32, 8);
    if (pb.d == 128 && pb.r == 64 && pb.p == 4) return PSF_AT(128, 64, 4);
    if (pb.d == 128 && pb.r == 32 && pb.p == 4) return PSF_AT(128, 32, 4);
    if (pb.d == 128 && pb.r == 64 && pb.p == 8) return PSF_AT(128, 64, 8);
    if (pb.d == 128 && pb.r == 32 && pb.p == 8) return PSF_AT(128, 32, 8);
#undef PSF_AT
    return PSF_ERR_UNSUPPORTED;
}

// Non-causal attention (Section 2.2) = the causal kernels on one "block" of all n tokens whose
// state every token reads: the state kernel accumulates that block, the output kernel skips
// its in-block phase.
static Problem noncausal_problem(const Problem &pb0)
{
    Problem pb = base_case_problem(pb0);
    pb.b = pb0.n;
    pb.t = 2;
    return pb;
}

size_t mfma_noncausal_workspace_bytes(const Problem &pb) { return carve(noncausal_problem(pb), nullptr).total; }

psf_status mfma_attn_noncausal(const Problem &pb0, const void *Q, const void *K, const void *V, const void *G,
                               void *O, void *ws, hipStream_t s, StageTimer *tm)
{
    const Problem pb = noncausal_problem(pb0);
#define PSF_AT(D_, R_, P_) (attn_impl<D_, R_, P_>(pb, Q, K, V, G, O, ws, s, tm, nullptr, nullptr, true))
    PSF_DISPATCH(PSF_AT);
#undef PSF_AT
}

}  // namespace psf
