// Backward pass on MFMA (bf16 storage, d = dv in {64, 128}, p in {4, 8}, r in {32, 64}, b % 256 == 0).
// Included inside the anonymous namespace of psf_mfma.hip, after the forward kernels it reuses.
//
// Gradient of the forward function of Sections 3, 3.1, 3.2 (the paper prints no formula; this is
// the chain rule through the definition).  With C_j = [v_j | 1], row_i = sum_j w_ij C_j,
// D_i = 1 + row_i[dv], o_i = row_i[0:dv] / D_i:
//     g_i = dO_i / D_i,  c_i = -<dO_i, o_i> / D_i,  dw_ij = <g_i, v_j> + c_i,  dV_j = sum_i w_ij g_i
// pairs inside a block:  w = <q, k>^p,        dq_i += sum_j dw_ij p <q_i, k_j>^(p-1) k_j   (dk alike)
// pairs across blocks:   w = <m(q), m(k)>^2,  dm(q_i) = 2 sum_j dw_ij <m(q_i), m(k_j)> m(k_j) (dm(k) alike)
// The cross-block sums are linear-time through the prefix states Z_l of Section 3.1 and their
// mirror R_l = sum over later blocks of phi'(q_i) [g_i | c_i]^T:
//     dm(q_i)[e] = 2 sum_{b,c} Z_l[e,b,c] m(q_i)[b] g_i[c]  +  2 c_i (S_l m(q_i))[e]
//     dm(k_j)[e] = 2 sum_{b,c} R_l[e,b,c] m(k_j)[b] v_j[c]  +  2 (Rc_l m(k_j))[e]
//     dV_j      +=   phi'(k_j)^T R_l            (the forward cross-block product with R in place of Z)
// where S_l / Rc_l are the ones-column parts of the states.  Finally dq_i += J_m(q_i)^T dm(q_i)
// through Algorithm 1 (p = 4: m = sqrt(1/r) (x G1) * (x G2), inside k_bwd_dm at d = 64; d = 128 and
// p = 8 (one more level of the recursion): k_bwd_sketch_rows).

template <int E>
__device__ __forceinline__ float pow_n(float x)
{
    float r = x;
#pragma unroll
    for (int e = 1; e < E; ++e) r *= x;
    return r;
}

// ---- g, c and the layouts of g ------------------------------------------------------------
// One wave per token octet, lane = value column.  G_rm: g as bf16 rows; G8: octets [rows/8][D][8];
// G8r: the same octets with the blocks of every unit in reverse order (input of the mirror
// state kernel, which then is the forward state kernel unchanged); Cc: c as fp32.
template <int D>
__global__ __launch_bounds__(kWg) void k_bwd_prep(const bf16_t *__restrict__ dO, const bf16_t *__restrict__ O,
                                                  const float *__restrict__ Den, bf16_t *__restrict__ G_rm,
                                                  bf16_t *__restrict__ G8, bf16_t *__restrict__ G8r,
                                                  float *__restrict__ Cc, int n, int b, int t)
{
    static_assert(D % 64 == 0, "D / 64 value columns per lane");
    constexpr int CL = D / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t oct = (size_t)blockIdx.x * 4 + wave, row0 = oct * 8;
    uint16_t gb[CL][8];
    float dot[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float inv = 1.0f / Den[row0 + j];
        dot[j] = 0.f;
#pragma unroll
        for (int cl = 0; cl < CL; ++cl) {
            const int col = 64 * cl + lane;
            const float d_o = bf16_to_f32(dO[(row0 + j) * D + col]);
            const float o = bf16_to_f32(O[(row0 + j) * D + col]);
            gb[cl][j] = f32_to_bf16(d_o * inv);
            dot[j] += d_o * o * inv;
            G_rm[(row0 + j) * D + col] = gb[cl][j];
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) dot[j] += __shfl_xor(dot[j], m);
        if (lane == j) Cc[row0 + j] = -dot[j];
    }
    const size_t u = row0 / n, pos = row0 % n;
    const size_t rpos = (size_t)(t - 1 - (int)(pos / b)) * b + pos % b;
#pragma unroll
    for (int cl = 0; cl < CL; ++cl) {
        const int col = 64 * cl + lane;
        uint4 pk;
        pk.x = gb[cl][0] | ((uint32_t)gb[cl][1] << 16);
        pk.y = gb[cl][2] | ((uint32_t)gb[cl][3] << 16);
        pk.z = gb[cl][4] | ((uint32_t)gb[cl][5] << 16);
        pk.w = gb[cl][6] | ((uint32_t)gb[cl][7] << 16);
        *(uint4 *)&G8[(oct * D + col) * 8] = pk;
        *(uint4 *)&G8r[(((u * n + rpos) >> 3) * D + col) * 8] = pk;
    }
}

// ---- m(Q) octets in reverse block order and the c-weighted partial sums --------------------
// Workgroup = 256 tokens: M8r [rows/8][2][R][4] fp32 (reverse block order) and
// Sc = sum_i c_i m_i m_i^T (R x R fp32) at the part's reverse-order position.
template <int R>
__global__ __launch_bounds__(kWg) void k_bwd_qoct(const bf16_t *__restrict__ MQ, const float *__restrict__ Cc,
                                                  float *__restrict__ M8r, float *__restrict__ ScPart, int n,
                                                  int b, int t)
{
    constexpr int OT = R / 32;
    __shared__ float red[4][32][33];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, x = lane & 31, h = lane >> 5;
    const size_t row0 = (size_t)blockIdx.x * 256;
    const size_t u = row0 / n, pos0 = row0 % n;
    const size_t rrow0 = u * n + (size_t)(t - 1 - (int)(pos0 / b)) * b + pos0 % b;
    f32x16 sacc[OT][OT];
#pragma unroll
    for (int i = 0; i < OT; ++i)
#pragma unroll
        for (int j = 0; j < OT; ++j) sacc[i][j] = f32x16{0};
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
        const size_t tile0 = row0 + wave * 64 + 32 * tt, rtile0 = rrow0 + wave * 64 + 32 * tt;
        // lane = sketch column 32 ot + x, register v = token 8 (v / 4) + 4 h + v % 4
        f32x16 m[OT], mw[OT];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const size_t tok = tile0 + 8 * (v / 4) + 4 * h + (v % 4);
            const float cw = Cc[tok];
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
                m[ot][v] = bf16_to_f32(MQ[tok * R + 32 * ot + x]);
                mw[ot][v] = m[ot][v] * cw;
            }
        }
#pragma unroll
        for (int ot = 0; ot < OT; ++ot)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 q4 = {m[ot][4 * gq], m[ot][4 * gq + 1], m[ot][4 * gq + 2], m[ot][4 * gq + 3]};
                const size_t oct = (rtile0 >> 3) + gq;
                *(f32x4 *)&M8r[((oct * 2 + h) * R + 32 * ot + x) * 4] = q4;
            }
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
            bf16x8 f[OT], fw[OT];
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
                f[ot] = cvt8_from16(m[ot], 8 * sp);
                fw[ot] = cvt8_from16(mw[ot], 8 * sp);
            }
#pragma unroll
            for (int i = 0; i < OT; ++i)
#pragma unroll
                for (int j = 0; j < OT; ++j) sacc[i][j] = mfma32(f[i], fw[j], sacc[i][j]);
        }
    }
    float *out = ScPart + (rrow0 / 256) * R * R;
#pragma unroll
    for (int i = 0; i < OT; ++i)
#pragma unroll
        for (int j = 0; j < OT; ++j) {
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave][8 * (v / 4) + 4 * h + (v % 4)][x] = sacc[i][j][v];
            __syncthreads();
            for (int idx = tid; idx < 32 * 32; idx += kWg) {
                const int a = idx / 32, c = idx % 32;
                out[(size_t)(32 * i + a) * R + 32 * j + c] = red[0][a][c] + red[1][a][c] + red[2][a][c] + red[3][a][c];
            }
        }
}

// ---- state snapshots re-laid for the gradient ------------------------------------------------
// In:  Zs [snap][a][b'/8][c][8], the format the state kernel writes (b' > a doubled, b' = a once,
//      b' < a zero).  Out: ZT [snap][b][c/8][e][8] = 2 Z[e][b][c], twice the full symmetric state
//      (so only the diagonal needs arithmetic) with the value column as the contraction octet and
//      the free sketch index e as the row of an MFMA A operand.  Workgroup = (octet of b, snapshot).
// DC value columns per workgroup (blockIdx.z picks the range): D = 128 goes in two halves so that
// two workgroups fit a CU.
template <int R, int D, int DC = D>
__global__ __launch_bounds__(kWg) void k_bwd_relayout(const bf16_t *__restrict__ Zs, bf16_t *__restrict__ ZT)
{
    static_assert(DC >= 64 && D % DC == 0, "the swizzle needs eight column octets");
    // [b % 8][e][c], the 16-byte column c / 8 of row e stored at (c / 8) ^ (e % 8): the final
    // reads walk e with a fixed column and would otherwise all hit the same banks
    __shared__ __attribute__((aligned(16))) bf16_t F[8][R][DC];
    auto at = [&](int b8, int e, int c) -> bf16_t & { return F[b8][e][(((c >> 3) ^ (e & 7)) << 3) + (c & 7)]; };
    const int tid = threadIdx.x, ob = blockIdx.x, c0 = blockIdx.z * DC;
    const bf16_t *src = Zs + (size_t)blockIdx.y * R * R * D;
    bf16_t *dst = ZT + (size_t)blockIdx.y * R * R * D;
    auto twice = [](uint32_t bits) { return f32_to_bf16(2.0f * bf16_to_f32((bf16_t)bits)); };
    // 16-byte pieces of the source, all loads of a thread issued before their use:
    //   pieces [0, 8 ob DC): rows e < 8 ob, octet ob (b > e there: 2 Z[e][b][c] = Zs[e][b][c])
    //   the rest: rows a of this octet, column octets ob2 >= ob
    constexpr int PIECES = 8 * DC * (R / 8) / kWg;
    const int n_a = 8 * ob * DC, per_a = (R / 8 - ob) * DC;
    uint4 pk[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
        const int idx = tid + i * kWg;
        size_t off;
        if (idx < n_a) {
            off = ((size_t)(idx / DC) * (R / 8) + ob) * D + c0 + idx % DC;
        } else {
            const int k2 = idx - n_a, a8 = k2 / per_a, rem = k2 % per_a;
            off = ((size_t)(8 * ob + a8) * (R / 8) + ob + rem / DC) * D + c0 + rem % DC;
        }
        pk[i] = *(const uint4 *)&src[off * 8];
    }
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
        const int idx = tid + i * kWg;
        const uint32_t w[4] = {pk[i].x, pk[i].y, pk[i].z, pk[i].w};
        if (idx < n_a) {
            const int e = idx / DC, c = idx % DC;
#pragma unroll
            for (int j = 0; j < 8; ++j) at(j, e, c) = (bf16_t)((w[j / 2] >> (16 * (j % 2))) & 0xffffu);
        } else {
            const int k2 = idx - n_a, a8 = k2 / per_a, rem = k2 % per_a, ob2 = ob + rem / DC, c = rem % DC;
            const int a = 8 * ob + a8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int bp = 8 * ob2 + j;
                const uint32_t bits = (w[j / 2] >> (16 * (j % 2))) & 0xffffu;
                if (bp > a) {
                    at(a8, bp, c) = (bf16_t)bits;          // (b = a, e = b')
                    if (ob2 == ob) at(j, a, c) = (bf16_t)bits;   // mirror inside the diagonal octet: (b = b', e = a)
                } else if (bp == a) {
                    at(a8, a, c) = twice(bits);
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
        const int idx = tid + i * kWg;
        const int b8 = idx / ((DC / 8) * R), c8 = (idx / R) % (DC / 8), e = idx % R;
        *(uint4 *)&dst[((((size_t)(8 * ob + b8)) * (D / 8) + c0 / 8 + c8) * R + e) * 8] = *(const uint4 *)&F[b8][e][8 * (c8 ^ (e & 7))];
    }
}

// ---- through Algorithm 1 (p = 4), one 32-token tile of a wave --------------------------------
// dx = dXacc (if ADD_BASE) + sqrt(1/r) [(dm * (x G2)) G1^T + (dm * (x G1)) G2^T].  lds: the transposed sketch
// matrices as the forward sketch kernel stages them (for the recomputed projections); go: G1,
// G2 as given, rows [d][r] padded to GP (for the transposed products, whose A fragments are read
// in accumulator order).  dm: lane = token, register = sketch column, as the accumulators of
// the cross-block kernel leave it.
template <int D, int R, bool ADD_BASE = true>
__device__ __forceinline__ void sketch_grad_tile(const SketchLds<D, R> &lds, const bf16_t *go,
                                                 const bf16_t *__restrict__ X, const f32x16 *dm,
                                                 const float *__restrict__ dXacc, bf16_t *__restrict__ dX,
                                                 size_t row, int x, int h)
{
    constexpr int KS = D / 16, NT = R / 32, DT = D / 32, GP = R + 8;
    const float scale = sqrtf(1.0f / (float)R);
    bf16x8 xfr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) xfr[s] = *(const bf16x8 *)&X[row * D + 16 * s + 8 * h];
    f32x16 a0[NT], a1[NT];                                  // lane = token, register = sketch column
    project<D, R, KS, true>(lds.gt[0], xfr, a0, x, h);
    project<D, R, KS, true>(lds.gt[1], xfr, a1, x, h);
    bf16x8 d0[2 * NT], d1[2 * NT];                          // B operands, contraction over sketch columns
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        f32x16 da0, da1;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            da0[v] = scale * dm[ct][v] * a1[ct][v];
            da1[v] = scale * dm[ct][v] * a0[ct][v];
        }
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
            d0[2 * ct + sp] = cvt8_from16(da0, 8 * sp);
            d1[2 * ct + sp] = cvt8_from16(da1, 8 * sp);
        }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        f32x16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < 2 * NT; ++ks) {
            // entries e of the step are sketch columns 16 ks + 8 (e / 4) + 4 h + e % 4
            const int off = (32 * dt + x) * GP + 16 * ks + 4 * h;
            const bf16x4 lo1 = *(const bf16x4 *)&go[off], hi1 = *(const bf16x4 *)&go[off + 8];
            const bf16x4 lo2 = *(const bf16x4 *)&go[D * GP + off], hi2 = *(const bf16x4 *)&go[D * GP + off + 8];
            bf16x8 f1, f2;
#pragma unroll
            for (int e = 0; e < 4; ++e) { f1[e] = lo1[e]; f1[4 + e] = hi1[e]; f2[e] = lo2[e]; f2[4 + e] = hi2[e]; }
            acc = mfma32(f1, d0[ks], acc);
            acc = mfma32(f2, d1[ks], acc);
        }
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const size_t off = row * D + 32 * dt + 8 * gq + 4 * h;
            f32x4 q4 = {acc[4 * gq], acc[4 * gq + 1], acc[4 * gq + 2], acc[4 * gq + 3]};
            if constexpr (ADD_BASE) {
                const f32x4 base = *(const f32x4 *)&dXacc[off];
#pragma unroll
                for (int j = 0; j < 4; ++j) q4[j] += base[j];
            }
            *(bf16x4 *)&dX[off] = cvt4(q4);
        }
    }
}

// Both sets of sketch matrices of one parameter set into LDS (see sketch_grad_tile).
template <int D, int R>
__device__ __forceinline__ void sketch_grad_stage(SketchLds<D, R> &lds, bf16_t *go, const bf16_t *__restrict__ Gt,
                                                  const bf16_t *__restrict__ G)
{
    constexpr int GP = R + 8;
    stage_gt<D, R, D>(lds.gt[0], Gt);
    stage_gt<D, R, D>(lds.gt[1], Gt + (size_t)D * R);
    for (int idx = threadIdx.x; idx < 2 * D * (R / 8); idx += kWg) {
        const int m = idx / (D * (R / 8)), rem = idx % (D * (R / 8)), e = rem / (R / 8), part = rem % (R / 8);
        *(uint4 *)&go[(m * D + e) * GP + 8 * part] = *(const uint4 *)&G[(size_t)m * D * R + (size_t)e * R + 8 * part];
    }
}

// ---- through Algorithm 1 as a pass of its own (d = 128 or degree 8) ---------------------------
// dX = bf16(dXacc + J_m(x)^T dm) for 128 rows per workgroup (one 32-row tile per wave, lane = row), dm
// given as fp32 rows.  Degree 4: sketch_grad_tile.  Degree 8, with u_k = x G_k (k < 4),
// n1 = s u0 * u1, n2 = s u2 * u3, w1 = n1 G4, w2 = n2 G5, m = s w1 * w2, s = sqrt(1/r):
//     dw1 = s dm * w2, dw2 = s dm * w1;  dn1 = dw1 G4^T, dn2 = dw2 G5^T;
//     du0 = s dn1 * u1, du1 = s dn1 * u0, du2 = s dn2 * u3, du3 = s dn2 * u2;  dx = sum_k du_k G_k^T.
// The matrices go through LDS in phases (two transposed ones for the projections, two as given
// for the transposed products at a time), as in the forward sketch kernel.
template <int D, int R, int P>
__global__ __launch_bounds__(kWg, 2) void k_bwd_sketch_rows(const bf16_t *__restrict__ X, const bf16_t *__restrict__ Gt,
                                                           const bf16_t *__restrict__ G, const float *__restrict__ dM,
                                                           const float *__restrict__ dXacc, bf16_t *__restrict__ dX,
                                                           int n, int heads, int per_head, size_t g_len)
{
    constexpr int KS = D / 16, NT = R / 32, RS = R / 16, DT = D / 32, GP = R + 8;
    __shared__ __attribute__((aligned(16))) SketchLds<D, R> lds;
    __shared__ __attribute__((aligned(16))) bf16_t go[2 * D * GP];
    const int tid = threadIdx.x, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t row0 = (size_t)blockIdx.x * 128, row = row0 + wave * 32 + x;
    const size_t goff = per_head ? (size_t)((row0 / n) % heads) * g_len : 0;
    const bf16_t *gt = Gt + goff, *g = G + goff;
    // dm of the tile: lane = row, register v of tile ct = sketch column 32 ct + 8 (v / 4) + 4 h + v % 4
    f32x16 dm[NT];
#pragma unroll
    for (int ct = 0; ct < NT; ++ct)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const f32x4 d4 = *(const f32x4 *)&dM[row * R + 32 * ct + 8 * gq + 4 * h];
#pragma unroll
            for (int j = 0; j < 4; ++j) dm[ct][4 * gq + j] = d4[j];
        }
    if constexpr (P == 4) {
        sketch_grad_stage<D, R>(lds, go, gt, g);
        __syncthreads();
        sketch_grad_tile<D, R, true>(lds, go, X, dm, dXacc, dX, row, x, h);
    } else {
        static_assert(P == 8, "degree 4 or 8");
        const float scale = sqrtf(1.0f / (float)R);
        // rows [0, nrows) of a matrix given as [nrows][R] -> go[which] with rows padded to GP
        auto stage_rows = [&](int which, const bf16_t *src, int nrows) {
            for (int idx = tid; idx < nrows * (R / 8); idx += kWg) {
                const int e = idx / (R / 8), part = idx % (R / 8);
                *(uint4 *)&go[(which * D + e) * GP + 8 * part] = *(const uint4 *)&src[(size_t)e * R + 8 * part];
            }
        };
        // out[i][row] = sum_k M[i][k] v[k][row], M as given ([.][R], staged by stage_rows), v as B
        // fragments in accumulator order (entries e of step ks: k = 16 ks + 8 (e / 4) + 4 h + e % 4)
        auto times_rows = [&](int which, int tile, const bf16x8 *v, f32x16 acc) {
#pragma unroll
            for (int ks = 0; ks < RS; ++ks) {
                const int off = (which * D + 32 * tile + x) * GP + 16 * ks + 4 * h;
                const bf16x4 lo = *(const bf16x4 *)&go[off], hi = *(const bf16x4 *)&go[off + 8];
                bf16x8 f;
#pragma unroll
                for (int e = 0; e < 4; ++e) { f[e] = lo[e]; f[4 + e] = hi[e]; }
                acc = mfma32(f, v[ks], acc);
            }
            return acc;
        };
        auto to_frags = [&](const f32x16 (&a)[NT], bf16x8 (&f)[RS]) {
#pragma unroll
            for (int ct = 0; ct < NT; ++ct)
#pragma unroll
                for (int q2 = 0; q2 < 2; ++q2) f[2 * ct + q2] = cvt8_from16(a[ct], 8 * q2);
        };
        bf16x8 xfr[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) xfr[s] = *(const bf16x8 *)&X[row * D + 16 * s + 8 * h];
        // the projections are kept as bf16 (like every operand of the products they enter): half the registers
        bf16x8 ub[4][RS];
        bf16x8 nfr[2][RS];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            __syncthreads();
            stage_gt<D, R, D>(lds.gt[0], gt + (size_t)(2 * half) * D * R);
            stage_gt<D, R, D>(lds.gt[1], gt + (size_t)(2 * half + 1) * D * R);
            __syncthreads();
            f32x16 ua[NT], uc[NT];
            project<D, R, KS, true>(lds.gt[0], xfr, ua, x, h);
            project<D, R, KS, true>(lds.gt[1], xfr, uc, x, h);
            f32x16 nn[NT];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) nn[ct] = scale * (ua[ct] * uc[ct]);
            to_frags(nn, nfr[half]);
            to_frags(ua, ub[2 * half]);
            to_frags(uc, ub[2 * half + 1]);
        }
        auto u_at = [&](int k, int ct, int v) { return (float)ub[k][2 * ct + v / 8][v % 8]; };
        __syncthreads();
        const size_t inner = (size_t)4 * D * R;
        stage_gt<D, R, R>(lds.gt[0], gt + inner);
        stage_gt<D, R, R>(lds.gt[1], gt + inner + (size_t)R * R);
        stage_rows(0, g + inner, R);
        stage_rows(1, g + inner + (size_t)R * R, R);
        __syncthreads();
        bf16x8 duf[4][RS];
        {
            f32x16 w1[NT], w2[NT];
            project_inner<D, R, true>(lds.gt[0], nfr[0], w1, x, h);
            project_inner<D, R, true>(lds.gt[1], nfr[1], w2, x, h);
            f32x16 d1[NT], d2[NT];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                d1[ct] = scale * (dm[ct] * w2[ct]);
                d2[ct] = scale * (dm[ct] * w1[ct]);
            }
            bf16x8 dw1[RS], dw2[RS];
            to_frags(d1, dw1);
            to_frags(d2, dw2);
            f32x16 t0[NT], t1[NT];
#pragma unroll
            for (int ct = 0; ct < NT; ++ct) {
                const f32x16 dn1 = times_rows(0, ct, dw1, f32x16{0}), dn2 = times_rows(1, ct, dw2, f32x16{0});
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    t0[ct][v] = scale * dn1[v] * u_at(1, ct, v);
                    t1[ct][v] = scale * dn1[v] * u_at(0, ct, v);
                    d1[ct][v] = scale * dn2[v] * u_at(3, ct, v);
                    d2[ct][v] = scale * dn2[v] * u_at(2, ct, v);
                }
            }
            to_frags(t0, duf[0]);
            to_frags(t1, duf[1]);
            to_frags(d1, duf[2]);
            to_frags(d2, duf[3]);
        }
        f32x16 dx[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) dx[dt] = f32x16{0};
#pragma unroll
        for (int pair = 0; pair < 2; ++pair) {
            __syncthreads();
            stage_rows(0, g + (size_t)(2 * pair) * D * R, D);
            stage_rows(1, g + (size_t)(2 * pair + 1) * D * R, D);
            __syncthreads();
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                dx[dt] = times_rows(0, dt, duf[2 * pair], dx[dt]);
                dx[dt] = times_rows(1, dt, duf[2 * pair + 1], dx[dt]);
            }
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const size_t off = row * D + 32 * dt + 8 * gq + 4 * h;
                const f32x4 base = *(const f32x4 *)&dXacc[off];
                const f32x4 q4 = {dx[dt][4 * gq] + base[0], dx[dt][4 * gq + 1] + base[1], dx[dt][4 * gq + 2] + base[2],
                                  dx[dt][4 * gq + 3] + base[3]};
                *(bf16x4 *)&dX[off] = cvt4(q4);
            }
    }
}

// ---- generic cross-block contraction ---------------------------------------------------------
// out^T[o][token] += sum_{a < NS} sum_{k < NV} (sc_token[a] * vec_token[k]) * Z[a][k][o],  Z stored
// [NS][NV/8][NO][8] bf16 (k octets innermost: 16-byte A fragments with rows o).  The B operand
// (the products) is generated in registers from the token's scalar sc[a] and its vector vec[.],
// which the caller holds as fp32 in contraction order (element e of step s = index 16 s + 8 h + e).
// SYM: Z carries the symmetry weights of the state kernel, steps below 16 (a / 16) are skipped.
// Workgroup = 128 TT tokens; rows of Z stream through LDS in chunks of ZA, double buffered.
template <int NS, int NV, int NO, bool SYM, int TT>
struct Cross {
    static constexpr int CT = NO / 32, VS = NV / 16;
    static constexpr int Z_PER = NV * NO;                      // bf16 elements per scalar index
    static constexpr int ZA = 16384 / Z_PER;                   // scalar indices per chunk (32 KB)
    static constexpr int CHUNK_BYTES = ZA * Z_PER * 2;
    static constexpr int NCHUNK = NS / ZA;
    static constexpr int LDS_BYTES = 2 * CHUNK_BYTES;
    static constexpr int DMA = CHUNK_BYTES / 16 / kWg;
    static_assert(ZA >= 1 && ZA <= 8 && 16 % ZA == 0 && NS % ZA == 0, "chunking");
    typedef __bf16 scvec __attribute__((ext_vector_type(ZA)));

    // sc_rows: bf16 rows [tokens][NS] of the workgroup's first token
    static __device__ __forceinline__ void run(const bf16_t *__restrict__ sc_rows, const f32x8 (&vec)[TT][VS],
                                               const bf16_t *__restrict__ Z, f32x16 (&out)[TT][CT],
                                               unsigned char *stage)
    {
        const int tid = threadIdx.x, lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int x = lane & 31, h = lane >> 5;
        auto copy_chunk = [&](int buf, int chunk) {
            const bf16_t *src = Z + (size_t)chunk * ZA * Z_PER;
#pragma unroll
            for (int q = 0; q < DMA; ++q)
                dma16(src + (size_t)(q * kWg + tid) * 8, stage + buf * CHUNK_BYTES + (size_t)(q * kWg + wave * 64) * 16);
        };
        auto load_sc = [&](int chunk, scvec (&dst)[TT]) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                dst[tt] = *(const scvec *)&sc_rows[(size_t)(wave * 32 * TT + 32 * tt + x) * NS + chunk * ZA];
        };
        scvec sc[TT], sc_next[TT];
        copy_chunk(0, 0);
        load_sc(0, sc);
#pragma unroll 1
        for (int chunk = 0; chunk < NCHUNK; ++chunk) {
            const int buf = chunk & 1;
            wait_vmem_le<0>();
            __syncthreads();                               // chunk landed; the other buffer is free
            if (chunk + 1 < NCHUNK) {
                copy_chunk(buf ^ 1, chunk + 1);
                load_sc(chunk + 1, sc_next);
            }
            const bf16_t *zc = (const bf16_t *)(stage + buf * CHUNK_BYTES);
            const int s0 = SYM ? (chunk * ZA) / 16 : 0;
#pragma unroll
            for (int ai = 0; ai < ZA; ++ai) {
                const bf16_t *za = zc + ai * Z_PER;
#pragma unroll
                for (int s = 0; s < VS; ++s) {
                    if (s < s0) continue;
                    bf16x8 zf[CT];
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) zf[ct] = *(const bf16x8 *)&za[((2 * s + h) * NO + 32 * ct + x) * 8];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) {
                        const float ma = (float)sc[tt][ai];
                        f32x8 pr;
#pragma unroll
                        for (int e = 0; e < 8; ++e) pr[e] = ma * vec[tt][s][e];
                        const bf16x8 frag = cvt8(pr);
#pragma unroll
                        for (int ct = 0; ct < CT; ++ct) out[tt][ct] = mfma32(zf[ct], frag, out[tt][ct]);
                    }
                }
            }
            if (chunk + 1 < NCHUNK) {
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) sc[tt] = sc_next[tt];
            }
        }
        __syncthreads();                                   // the caller may reuse the stage
    }
};

// ---- dm(q) and dm(k): cross-block part -------------------------------------------------------
// QSIDE: tokens of block l >= 1 with ZT / S of slot l - 1, vec = g, coefficient c_i.
// key side: tokens of block l <= t - 2 with RT / Rc of the mirror slot t - 2 - l, vec = v,
// coefficient 1.  Blocks without a cross-block term have dm = 0.  dm stays in registers and goes
// straight through Algorithm 1 (sketch_grad_tile): dX = bf16(dXacc + J_m(x)^T dm), with dXacc the
// in-block part, for the rows X (Q or K) of the workgroup.
// LS (in-block rule of Section 3.1, R == D): the in-block weights are functions of the sketches
// too, so dXacc holds the in-block part of dm ([rows][R] fp32), which joins dm before the sketch:
// dX = bf16(J_m(x)^T (dm + dXacc)).
// RAW (learned sketches): dm itself is the result, fp32 rows [rows][R] in dMout (no sketch matrices).
template <int R, int D, bool QSIDE, int TT, bool LS = false, bool RAW = false>
__global__ __launch_bounds__(kWg, 2) void k_bwd_dm(const bf16_t *__restrict__ M, const bf16_t *__restrict__ Vec,
                                                  const float *__restrict__ Cc, const bf16_t *__restrict__ ZT,
                                                  const bf16_t *__restrict__ Shi, const bf16_t *__restrict__ Slo,
                                                  const bf16_t *__restrict__ Xrows, const bf16_t *__restrict__ Gt,
                                                  const bf16_t *__restrict__ G, const float *__restrict__ dXacc,
                                                  bf16_t *__restrict__ dX, int n, int b, int t, int heads,
                                                  int per_head, size_t g_len, float *__restrict__ dMout = nullptr)
{
    using X = Cross<R, D, R, false, TT>;
    static_assert(RAW || sizeof(SketchLds<D, R>) + 2 * D * (R + 8) * 2 <= X::LDS_BYTES, "the sketch matrices reuse the stage");
    constexpr int AT = R / 32, RS = R / 16, VS = D / 16, TOK_WG = 128 * TT;
    __shared__ __attribute__((aligned(16))) unsigned char stage[X::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_per_unit = n / TOK_WG;
    int wg = blockIdx.x;                                    // XCD-aware order: one state snapshot, one L2
    if ((gridDim.x & 7) == 0) wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int u = wg / tiles_per_unit, i0 = (wg % tiles_per_unit) * TOK_WG;
    const int l = i0 / b;
    const size_t urow = (size_t)u * n;
    const bool has = QSIDE ? l > 0 : l < t - 1;
    const int slot = QSIDE ? l - 1 : t - 2 - l;

    f32x16 out[TT][AT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int at = 0; at < AT; ++at) out[tt][at] = f32x16{0};
    if (has) {
        f32x8 vec[TT][VS];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int s = 0; s < VS; ++s) {
                const bf16x8 raw = *(const bf16x8 *)&Vec[(urow + i0 + wave * 32 * TT + 32 * tt + x) * D + 16 * s + 8 * h];
#pragma unroll
                for (int e = 0; e < 8; ++e) vec[tt][s][e] = (float)raw[e];
            }
        X::run(M + (urow + i0) * R, vec, ZT + ((size_t)u * (t - 1) + slot) * R * R * D, out, stage);

        // ones column: (S m)[a] per token with S as hi + lo A operands [b'/8][a][8]
        bf16x8 mfr[TT][RS];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int s = 0; s < RS; ++s)
                mfr[tt][s] = *(const bf16x8 *)&M[(urow + i0 + wave * 32 * TT + 32 * tt + x) * R + 16 * s + 8 * h];
        const size_t sbase = ((size_t)u * (t - 1) + slot) * R * R;
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
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const float coef = QSIDE ? Cc[urow + i0 + wave * 32 * TT + 32 * tt + x] : 1.0f;
#pragma unroll
                for (int v = 0; v < 16; ++v) out[tt][at][v] += 2.0f * coef * td[tt][v];   // the state operand is stored doubled
            }
        }
    }
    if constexpr (RAW) {
        // register v of out[tt][at]: sketch column 32 at + 8 (v / 4) + 4 h + v % 4
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int at = 0; at < AT; ++at)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const f32x4 o4 = {out[tt][at][4 * gq], out[tt][at][4 * gq + 1], out[tt][at][4 * gq + 2],
                                      out[tt][at][4 * gq + 3]};
                    *(f32x4 *)&dMout[(urow + i0 + wave * 32 * TT + 32 * tt + x) * R + 32 * at + 8 * gq + 4 * h] = o4;
                }
        return;
    }
    // through the sketch; the stage is free again (the contraction ends with a barrier)
    SketchLds<D, R> &lds = *(SketchLds<D, R> *)stage;
    bf16_t *go = (bf16_t *)(stage + sizeof(SketchLds<D, R>));
    const size_t goff = per_head ? (size_t)(u % heads) * g_len : 0;
    sketch_grad_stage<D, R>(lds, go, Gt + goff, G + goff);
    __syncthreads();
    if constexpr (LS) {
        static_assert(R == D, "the in-block kernels leave dm in the layout of a gradient row");
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int at = 0; at < AT; ++at)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    // register v of out[tt][at]: sketch column 32 at + 8 (v / 4) + 4 h + v % 4
                    const f32x4 a4 = *(const f32x4 *)&dXacc[(urow + i0 + wave * 32 * TT + 32 * tt + x) * R + 32 * at +
                                                            8 * gq + 4 * h];
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[tt][at][4 * gq + j] += a4[j];
                }
    }
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
        sketch_grad_tile<D, R, !LS>(lds, go, Xrows, out[tt], dXacc, dX, urow + i0 + wave * 32 * TT + 32 * tt + x, x,
                                    h);
}

// ---- dV: cross-block part = phi'(k_j)^T R_l (value columns) ----------------------------------
template <int R, int D, int TT>
__global__ __launch_bounds__(kWg, 2) void k_bwd_dvc(const bf16_t *__restrict__ MK, const bf16_t *__restrict__ Rg,
                                                   float *__restrict__ dVc, int n, int b, int t)
{
    using X = Cross<R, R, D, true, TT>;
    constexpr int CT = D / 32, RS = R / 16, TOK_WG = 128 * TT;
    __shared__ __attribute__((aligned(16))) unsigned char stage[X::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_per_unit = n / TOK_WG;
    int wg = blockIdx.x;                                    // XCD-aware order: one state snapshot, one L2
    if ((gridDim.x & 7) == 0) wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int u = wg / tiles_per_unit, i0 = (wg % tiles_per_unit) * TOK_WG;
    const int l = i0 / b;
    const size_t urow = (size_t)u * n;
    f32x16 out[TT][CT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) out[tt][ct] = f32x16{0};
    if (l < t - 1) {
        f32x8 vec[TT][RS];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int s = 0; s < RS; ++s) {
                const bf16x8 raw = *(const bf16x8 *)&MK[(urow + i0 + wave * 32 * TT + 32 * tt + x) * R + 16 * s + 8 * h];
#pragma unroll
                for (int e = 0; e < 8; ++e) vec[tt][s][e] = (float)raw[e];
            }
        X::run(MK + (urow + i0) * R, vec, Rg + ((size_t)u * (t - 1) + (t - 2 - l)) * R * R * D, out, stage);
    }
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const size_t row = urow + i0 + wave * 32 * TT + 32 * tt + x;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 q4 = {out[tt][ct][4 * gq], out[tt][ct][4 * gq + 1], out[tt][ct][4 * gq + 2],
                                  out[tt][ct][4 * gq + 3]};
                *(f32x4 *)&dVc[row * D + 32 * ct + 8 * gq + 4 * h] = q4;
            }
    }
}

// ---- in-block pairs ---------------------------------------------------------------------------
// Both kernels: workgroup = 32 NW "own" rows (wave = 32, held in registers as B operands), the
// other side streams through LDS in tiles of 64 rows, double buffered: its rows as
// [D/8][64][8] (16-byte A fragments, contraction over d) and its octets [8][D][8] (A fragments
// with contraction over the tile's rows).  Score tiles come out transposed (lane = own row,
// registers = streamed rows), are turned into bf16 B operands with one half-wave swap per
// register pair (as in the forward output kernel) and contracted with the octets.
constexpr int kLocT = 64;                                   // streamed rows per tile
// bytes of one [D/8][64][8] / [8][D][8] array
__host__ __device__ constexpr int loc_rows_bytes(int d) { return kLocT * d * 2; }

// X [rows][D] bf16 -> XF [rows/64][D/8][64][8]: per 64-row tile the layout the in-block kernels keep
// in LDS (16-byte A fragments with contraction over the D columns), so that staging a tile is
// a straight, fully coalesced copy.  d8 = D / 8.
// scale: a power of two (exact in bf16) the copy is multiplied by; 1 for a plain re-layout.
__global__ __launch_bounds__(kWg) void k_bwd_row_tiles(const bf16_t *__restrict__ X, bf16_t *__restrict__ XF,
                                                       size_t pieces, float scale, int d8)
{
    const size_t idx = (size_t)blockIdx.x * kWg + threadIdx.x;         // (tile, row, column octet)
    if (idx >= pieces) return;
    const size_t per_tile = (size_t)kLocT * d8, tile = idx / per_tile;
    const int key = (int)(idx % per_tile) / d8, doct = (int)(idx % d8);
    bf16x8 v = *(const bf16x8 *)&X[idx * 8];
    if (scale != 1.0f) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (__bf16)((float)v[e] * scale);
    }
    *(bf16x8 *)&XF[((tile * d8 + doct) * kLocT + key) * 8] = v;
}
// tile of rows [j0, j0 + 64) of XF -> LDS, straight copy
template <int NTHR, int D>
__device__ __forceinline__ void loc_stage_rows(const bf16_t *XF, size_t j0, unsigned char *dst, int tid, int wave)
{
#pragma unroll
    for (int q = 0; q < loc_rows_bytes(D) / 16 / NTHR; ++q)
        dma16(XF + j0 * D + (size_t)(q * NTHR + tid) * 8, dst + (size_t)(q * NTHR + wave * 64) * 16);
}
// octets of rows [j0, j0 + 64) of X8 ([rows/8][D][8]) -> LDS, straight copy
template <int NTHR, int D>
__device__ __forceinline__ void loc_stage_octets(const bf16_t *X8, size_t j0, unsigned char *dst, int tid, int wave)
{
#pragma unroll
    for (int q = 0; q < loc_rows_bytes(D) / 16 / NTHR; ++q)
        dma16(X8 + j0 * D + (size_t)(q * NTHR + tid) * 8, dst + (size_t)(q * NTHR + wave * 64) * 16);
}
// 16 fp32 (lane = own row, register v = streamed row 8 (v / 4) + 4 h + v % 4) -> two bf16 B
// fragments whose 8 entries are the streamed rows 16 sp + 8 h + e
__device__ __forceinline__ void loc_pack(const f32x16 &w, bf16x8 (&pw)[2])
{
#pragma unroll
    for (int sp = 0; sp < 2; ++sp) {
        uint4 u = __builtin_bit_cast(uint4, cvt8_from16(w, 8 * sp));
        const auto s0 = __builtin_amdgcn_permlane32_swap(u.x, u.z, false, false);
        const auto s1 = __builtin_amdgcn_permlane32_swap(u.y, u.w, false, false);
        u.x = s0[0]; u.z = s0[1]; u.y = s1[0]; u.w = s1[1];
        pw[sp] = __builtin_bit_cast(bf16x8, u);
    }
}

// dQ (in-block): own rows = queries, streamed = keys of the same block up to the diagonal.
//   dq_i = sum_{j <= i} (<g_i, v_j> + c_i) p <q_i, k_j>^(p-1) k_j          -> dQacc fp32 rows
template <int P, int NW, int D = 64>
__global__ __launch_bounds__(64 * NW, D == 64 ? 512 / (64 * NW) : 1) void k_bwd_local_q(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ KF,
                                                       const bf16_t *__restrict__ VF, const bf16_t *__restrict__ K8,
                                                       const bf16_t *__restrict__ G_rm, const float *__restrict__ Cc,
                                                       float *__restrict__ dQacc, int n, int b)
{
    constexpr int KS = D / 16, CT = D / 32, kLocRows = loc_rows_bytes(D), BUF = 3 * kLocRows, NTHR = 64 * NW, OWN = 32 * NW;
    __shared__ __attribute__((aligned(16))) unsigned char stage[2 * BUF];
    const int tid = threadIdx.x, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_per_unit = n / OWN;
    // XCD-aware order: consecutive workgroup ids go to different XCDs, so give each XCD a
    // contiguous range of tiles: the workgroups that stream the same rows then share one L2
    int wg = blockIdx.x;
    if ((gridDim.x & 7) == 0) wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int u = wg / tiles_per_unit, i0 = (wg % tiles_per_unit) * OWN;
    const int jb = (i0 / b) * b;
    const size_t urow = (size_t)u * n;
    const int tok0 = i0 + 32 * wave, tok = tok0 + x;
    bf16x8 qfr[KS], gfr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        qfr[s] = *(const bf16x8 *)&Q[(urow + tok) * D + 16 * s + 8 * h];
        gfr[s] = *(const bf16x8 *)&G_rm[(urow + tok) * D + 16 * s + 8 * h];
#pragma unroll
        for (int e = 0; e < 8; ++e) gfr[s][e] = (__bf16)((float)gfr[s][e] * (float)P);   // p of p s^(p-1), exact (power of two)
    }
    const float c_me = (float)P * Cc[urow + tok];
    f32x16 dq[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) dq[ct] = f32x16{0};
    const int ntiles = (i0 + OWN - jb) / kLocT;
    auto stage_tile = [&](int kt) {
        unsigned char *dst = stage + (kt & 1) * BUF;
        const size_t j0 = urow + jb + (size_t)kt * kLocT;
        loc_stage_rows<NTHR, D>(KF, j0, dst, tid, wave);
        loc_stage_rows<NTHR, D>(VF, j0, dst + kLocRows, tid, wave);
        loc_stage_octets<NTHR, D>(K8, j0, dst + 2 * kLocRows, tid, wave);
    };
    stage_tile(0);
#pragma unroll 1
    for (int kt = 0; kt < ntiles; ++kt) {
        wait_vmem_le<0>();
        __syncthreads();
        if (kt + 1 < ntiles) stage_tile(kt + 1);
        const bf16_t *ks = (const bf16_t *)(stage + (kt & 1) * BUF);
        const bf16_t *vs = ks + kLocRows / 2, *k8 = ks + kLocRows;
        if (jb + kt * kLocT <= tok0 + 31) {                // wave-uniform: some key of the tile is not later than every own token
            // both 32-key halves in one straight line: scores, then weights, then products
            f32x16 sc[2], dw[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                sc[sub] = f32x16{0};
                dw[sub] = f32x16{0};
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const bf16x8 kf = *(const bf16x8 *)&ks[((2 * s + h) * kLocT + 32 * sub + x) * 8];
                    const bf16x8 vf = *(const bf16x8 *)&vs[((2 * s + h) * kLocT + 32 * sub + x) * 8];
                    sc[sub] = mfma32(kf, qfr[s], sc[sub]);
                    dw[sub] = mfma32(vf, gfr[s], dw[sub]);
                }
            }
            bf16x8 pw[2][2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                // key = key0 + 8 (v / 4) + 4 h + v % 4 <= tok  <=>  8 (v / 4) + v % 4 <= lim
                const int lim = tok - (jb + kt * kLocT + 32 * sub) - 4 * h;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float sm = (8 * (v / 4) + (v % 4) <= lim) ? sc[sub][v] : 0.f;   // masked pairs: every power is 0
                    dw[sub][v] = (dw[sub][v] + c_me) * pow_n<P - 1>(sm);
                }
                loc_pack(dw[sub], pw[sub]);
            }
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int sp = 0; sp < 2; ++sp)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const bf16x8 kf8 = *(const bf16x8 *)&k8[((4 * sub + 2 * sp + h) * D + 32 * ct + x) * 8];
                        dq[ct] = mfma32(kf8, pw[sub][sp], dq[ct]);
                    }
        }
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const f32x4 q4 = {dq[ct][4 * gq], dq[ct][4 * gq + 1], dq[ct][4 * gq + 2], dq[ct][4 * gq + 3]};
            *(f32x4 *)&dQacc[(urow + tok) * D + 32 * ct + 8 * gq + 4 * h] = q4;
        }
}

// dK (in-block) and dV (in-block + the cross-block part already in dVc): own rows = keys,
// streamed = queries of the same block from the diagonal on.
//   dk_j = sum_{i >= j} (<g_i, v_j> + c_i) p <q_i, k_j>^(p-1) q_i   -> dKacc fp32 rows
//          (GF, the streamed rows of g for the first product, and the staged c carry the factor p)
//   dv_j = sum_{i >= j} <q_i, k_j>^p g_i + dVc_j                     -> dV bf16 rows
template <int P, int NW, int D = 64>
__global__ __launch_bounds__(64 * NW, D == 64 ? 512 / (64 * NW) : 1) void k_bwd_local_k(const bf16_t *__restrict__ QF, const bf16_t *__restrict__ K,
                                                       const bf16_t *__restrict__ V, const bf16_t *__restrict__ Q8,
                                                       const bf16_t *__restrict__ GF, const bf16_t *__restrict__ G8,
                                                       const float *__restrict__ Cc, const float *__restrict__ dVc,
                                                       float *__restrict__ dKacc, bf16_t *__restrict__ dV, int n,
                                                       int b)
{
    constexpr int KS = D / 16, CT = D / 32, kLocRows = loc_rows_bytes(D), BUF = 4 * kLocRows + kLocT * 4, NTHR = 64 * NW, OWN = 32 * NW;
    __shared__ __attribute__((aligned(16))) unsigned char stage[2 * BUF];
    const int tid = threadIdx.x, lane = tid & 63, x = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_per_unit = n / OWN;
    int wg = blockIdx.x;                                    // XCD-aware order, as in k_bwd_local_q
    if ((gridDim.x & 7) == 0) wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int u = wg / tiles_per_unit, j0 = (wg % tiles_per_unit) * OWN;
    const int jb = (j0 / b) * b;
    const size_t urow = (size_t)u * n;
    const int key0 = j0 + 32 * wave, key = key0 + x;
    bf16x8 kfr[KS], vfr[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        kfr[s] = *(const bf16x8 *)&K[(urow + key) * D + 16 * s + 8 * h];
        vfr[s] = *(const bf16x8 *)&V[(urow + key) * D + 16 * s + 8 * h];
    }
    f32x16 dk[CT], dv[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) dk[ct] = dv[ct] = f32x16{0};
    const int first = (j0 - jb) / kLocT, ntiles = b / kLocT;
    auto stage_tile = [&](int qt) {
        unsigned char *dst = stage + (qt & 1) * BUF;
        const size_t t0 = urow + jb + (size_t)qt * kLocT;
        loc_stage_rows<NTHR, D>(QF, t0, dst, tid, wave);
        loc_stage_rows<NTHR, D>(GF, t0, dst + kLocRows, tid, wave);
        loc_stage_octets<NTHR, D>(Q8, t0, dst + 2 * kLocRows, tid, wave);
        loc_stage_octets<NTHR, D>(G8, t0, dst + 3 * kLocRows, tid, wave);
        if (tid < kLocT) ((float *)(dst + 4 * kLocRows))[tid] = (float)P * Cc[t0 + tid];
    };
    stage_tile(first);
#pragma unroll 1
    for (int qt = first; qt < ntiles; ++qt) {
        wait_all_memory();
        __syncthreads();
        if (qt + 1 < ntiles) stage_tile(qt + 1);
        const bf16_t *qs = (const bf16_t *)(stage + (qt & 1) * BUF);
        const bf16_t *gs = qs + kLocRows / 2, *q8 = qs + kLocRows, *g8 = qs + 3 * (kLocRows / 2);
        const float *cs = (const float *)(stage + (qt & 1) * BUF + 4 * kLocRows);
        if (jb + qt * kLocT + kLocT - 1 >= key0) {         // wave-uniform: some token of the tile is not earlier than every own key
            f32x16 sc[2], dw[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                sc[sub] = f32x16{0};
                dw[sub] = f32x16{0};
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const bf16x8 qf = *(const bf16x8 *)&qs[((2 * s + h) * kLocT + 32 * sub + x) * 8];
                    const bf16x8 gf = *(const bf16x8 *)&gs[((2 * s + h) * kLocT + 32 * sub + x) * 8];
                    sc[sub] = mfma32(qf, kfr[s], sc[sub]);
                    dw[sub] = mfma32(gf, vfr[s], dw[sub]);
                }
            }
            bf16x8 pww[2][2], pwp[2][2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                // key <= token t0 + 8 gq + 4 h + j  <=>  8 gq + j >= lim
                const int lim = key - (jb + qt * kLocT + 32 * sub) - 4 * h;
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const f32x4 c4 = *(const f32x4 *)&cs[32 * sub + 8 * gq + 4 * h];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int v = 4 * gq + j;
                        const float sm = (8 * gq + j >= lim) ? sc[sub][v] : 0.f;   // masked pairs: every power is 0
                        const float pm1 = pow_n<P - 1>(sm);
                        sc[sub][v] = pm1 * sm;
                        dw[sub][v] = (dw[sub][v] + c4[j]) * pm1;      // g and c arrive multiplied by p
                    }
                }
                loc_pack(sc[sub], pww[sub]);
                loc_pack(dw[sub], pwp[sub]);
            }
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int sp = 0; sp < 2; ++sp)
#pragma unroll
                    for (int ct = 0; ct < CT; ++ct) {
                        const bf16x8 qf8 = *(const bf16x8 *)&q8[((4 * sub + 2 * sp + h) * D + 32 * ct + x) * 8];
                        const bf16x8 gf8 = *(const bf16x8 *)&g8[((4 * sub + 2 * sp + h) * D + 32 * ct + x) * 8];
                        dk[ct] = mfma32(qf8, pwp[sub][sp], dk[ct]);
                        dv[ct] = mfma32(gf8, pww[sub][sp], dv[ct]);
                    }
        }
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const size_t off = (urow + key) * D + 32 * ct + 8 * gq + 4 * h;
            const f32x4 k4 = {dk[ct][4 * gq], dk[ct][4 * gq + 1], dk[ct][4 * gq + 2], dk[ct][4 * gq + 3]};
            *(f32x4 *)&dKacc[off] = k4;
            const f32x4 c4 = *(const f32x4 *)&dVc[off];
            const f32x4 v4 = {dv[ct][4 * gq] + c4[0], dv[ct][4 * gq + 1] + c4[1], dv[ct][4 * gq + 2] + c4[2],
                              dv[ct][4 * gq + 3] + c4[3]};
            *(bf16x4 *)&dV[off] = cvt4(v4);
        }
}

// ---- host ---------------------------------------------------------------------------------------
struct MfmaBwdWs {
    void *fwd;                                               // the forward workspace
    bf16_t *O, *MK, *G_rm, *G8, *G8r, *Q8, *K8, *QF, *KF, *VF, *GF, *Rg, *ZT, *RT, *Rchi, *Rclo;
    float *Den, *Cc, *M8r, *ScPart, *dVc, *dQacc, *dKacc;
    // learned sketches: backward weight stream, what the row kernel leaves for the parameter
    // kernel (one side at a time), its workgroup sums, the per-unit parameter sums of both sides
    bf16_t *LB;
    LbStage sg;
    float *GB1, *part;
    size_t total;
};

MfmaBwdWs carve_bwd(const Problem &pb, void *ws)
{
    MfmaBwdWs w;
    const size_t rows = (size_t)pb.units * pb.n, R = pb.r, D = pb.d, tb = pb.t > 1 ? pb.t - 1 : 0;
    const size_t snaps = (size_t)pb.units * tb;
    size_t off = 0;
    char *base = (char *)ws;
    auto take = [&](size_t bytes) { char *p = base + off; off += align_up(bytes, 256); return (void *)p; };
    w.fwd = take(carve(pb, nullptr).total);
    w.O = (bf16_t *)take(rows * D * 2);
    w.MK = (bf16_t *)take(rows * R * 2);
    w.G_rm = (bf16_t *)take(rows * D * 2);
    w.G8 = (bf16_t *)take(rows * D * 2);
    w.G8r = (bf16_t *)take(rows * D * 2);
    w.Q8 = (bf16_t *)take(rows * D * 2);
    w.K8 = (bf16_t *)take(rows * D * 2);
    w.QF = (bf16_t *)take(rows * D * 2);
    w.KF = (bf16_t *)take(rows * D * 2);
    w.VF = (bf16_t *)take(rows * D * 2);
    w.GF = (bf16_t *)take(rows * D * 2);
    w.Rg = (bf16_t *)take(snaps * R * R * D * 2);
    w.ZT = (bf16_t *)take(snaps * R * R * D * 2);
    w.RT = (bf16_t *)take(snaps * R * R * D * 2);
    w.Rchi = (bf16_t *)take(snaps * R * R * 2);
    w.Rclo = (bf16_t *)take(snaps * R * R * 2);
    w.Den = (float *)take(rows * 4);
    w.Cc = (float *)take(rows * 4);
    w.M8r = (float *)take(rows * R * 4);
    w.ScPart = (float *)take(rows / 256 * R * R * 4);
    w.dVc = (float *)take(rows * D * 4);
    w.dQacc = (float *)take(rows * D * 4);
    w.dKacc = (float *)take(rows * D * 4);
    if (pb.learned) {
        const size_t sets = pb.per_head ? pb.heads : 1, nch = R / 4;
        w.LB = (bf16_t *)take(sets * 4 * nch * kLbSlot);
        w.sg.rows = rows;
        w.sg.XnR = (bf16_t *)take(rows * D * 2);
        w.sg.XnT = (bf16_t *)take(rows * D * 2);
        w.sg.A2R = (bf16_t *)take(2 * rows * R * 2);
        w.sg.A2T = (bf16_t *)take(2 * rows * R * 2);
        w.sg.DOR = (bf16_t *)take(2 * rows * R * 2);
        w.sg.DOT = (bf16_t *)take(2 * rows * R * 2);
        w.sg.DAR = (bf16_t *)take(2 * rows * R * 2);
        w.sg.DAT = (bf16_t *)take(2 * rows * R * 2);
        w.sg.ST = (float *)take(2 * 4 * rows * 4);
        w.GB1 = (float *)take(rows / 256 * 2 * 2 * D * 4);
        w.part = (float *)take(2 * (size_t)pb.units * learned_bwd_slices(pb) * pb.g_len * 4);
    }
    w.total = off;
    return w;
}

// What a forward call leaves for the backward pass when asked to (psf_causal_attn_fwd_save): its
// whole workspace (m(Q), the states Z_l and S_l, the transposed sketch matrices), the
// denominators and m(K) as bf16 rows.
struct MfmaSaved {
    void *fwd;
    float *Den;
    bf16_t *MK;
    size_t total;
};

MfmaSaved carve_saved(const Problem &pb, void *ptr)
{
    MfmaSaved sv;
    const size_t rows = (size_t)pb.units * pb.n;
    size_t off = 0;
    char *base = (char *)ptr;
    auto take = [&](size_t bytes) { char *p = base + off; off += align_up(bytes, 256); return (void *)p; };
    sv.fwd = take(carve(pb, nullptr).total);
    sv.Den = (float *)take(rows * 4);
    sv.MK = (bf16_t *)take(rows * pb.r * 2);
    sv.total = off;
    return sv;
}

// saved / O_saved: null = run the forward pass again inside; otherwise what psf_causal_attn_fwd_save
// left and the output it wrote.
template <int R, int D, int P>
psf_status attn_bwd_impl(const Problem &pb, const void *Q, const void *K, const void *V, const void *G,
                         const void *dO, void *dQ, void *dK, void *dV, void *ws, hipStream_t s, StageTimer *tm,
                         void *saved = nullptr, const void *O_saved = nullptr, float *dG = nullptr)
{
    constexpr int TT = D == 64 ? 2 : 1;                     // 32-token tiles per wave in the cross-block kernels
    constexpr int NWL = 4;                                  // waves per in-block workgroup: 256 own rows share a streamed tile
    MfmaBwdWs w = carve_bwd(pb, ws);
    MfmaWs f = carve(pb, w.fwd);
    const size_t rows = (size_t)pb.units * pb.n;
    const bf16_t *q = (const bf16_t *)Q, *k = (const bf16_t *)K, *v = (const bf16_t *)V;
    // in-block rule of Section 3.1 (r = d = 64 only): the in-block kernels take the sketches
    // m(Q), m(K) in place of Q, K with exponent 2 and leave the in-block part of dm
    const bool ls = !pb.local_exact;
    if (ls && !(R == D && P == 4)) return PSF_ERR_UNSUPPORTED;
    if (pb.learned && !(D == 64 && P == 4)) return PSF_ERR_UNSUPPORTED;
    if (pb.learned && ls) return PSF_ERR_UNSUPPORTED;
    psf_status st;
    if (saved) {
        const MfmaSaved sv = carve_saved(pb, saved);
        f = carve(pb, sv.fwd);
        w.Den = sv.Den;
        w.MK = sv.MK;
        w.O = (bf16_t *)O_saved;                           // read only
    } else {
        // forward pass again: O, the denominators, m(Q), m(K), the states Z_l and S_l
        st = attn_impl<D, R, P>(pb, Q, K, V, G, w.O, w.fwd, s, nullptr, w.Den, w.MK);
        if (st != PSF_OK) return st;
        if (pb.learned) {
            // (the learned key-side sketch kernel writes the state kernel's octets only)
            if (!learned_on_mfma(pb)) return PSF_ERR_UNSUPPORTED;
            const size_t count4 = rows * R / 4;
            hipLaunchKernelGGL((k_octets_to_rows<R>), dim3((unsigned)((count4 + kWg - 1) / kWg)), dim3(kWg), 0, s,
                               f.MK8, w.MK, count4);
            PSF_LAUNCH_CHECK();
        }
    }
    if (tm) tm->mark();
    const bf16_t *rq = ls ? f.MQ : q, *rk = ls ? w.MK : k;  // the rows the in-block weights are made of
    // g, c, layouts
    hipLaunchKernelGGL((k_bwd_prep<D>), dim3((unsigned)(rows / 32)), dim3(kWg), 0, s, (const bf16_t *)dO, w.O,
                       w.Den, w.G_rm, w.G8, w.G8r, w.Cc, pb.n, pb.b, pb.t);
    PSF_LAUNCH_CHECK();
    {
        const size_t octets = rows / 8;
        const unsigned grid = (unsigned)((octets * D + kWg - 1) / kWg);
        hipLaunchKernelGGL((k_v_octets<D>), dim3(grid), dim3(kWg), 0, s, rq, w.Q8, octets);
        PSF_LAUNCH_CHECK();
        hipLaunchKernelGGL((k_v_octets<D>), dim3(grid), dim3(kWg), 0, s, rk, w.K8, octets);
        PSF_LAUNCH_CHECK();
        const size_t pieces = rows * D / 8;
        const unsigned gridp = (unsigned)((pieces + kWg - 1) / kWg);
        const bf16_t *src[4] = {rq, rk, v, w.G_rm};
        bf16_t *dstf[4] = {w.QF, w.KF, w.VF, w.GF};
        for (int i = 0; i < 4; ++i) {
            // the copy of g that only feeds dW = <g, v> + c carries the factor e of d(s^e) = e s^(e-1) ds
            hipLaunchKernelGGL(k_bwd_row_tiles, dim3(gridp), dim3(kWg), 0, s, src[i], dstf[i], pieces,
                               i == 3 ? (ls ? 2.0f : (float)P) : 1.0f, D / 8);
            PSF_LAUNCH_CHECK();
        }
    }
    if (tm) tm->mark();
    // mirror states R_l (the forward state kernel on block-reversed inputs), re-laid states
    if (pb.t > 1) {
        hipLaunchKernelGGL((k_bwd_qoct<R>), dim3((unsigned)(rows / 256)), dim3(kWg), 0, s, f.MQ, w.Cc, w.M8r,
                           w.ScPart, pb.n, pb.b, pb.t);
        PSF_LAUNCH_CHECK();
        st = launch_state<D, R>(pb, w.M8r, w.G8r, w.Rg, s);
        if (st != PSF_OK) return st;
        hipLaunchKernelGGL((k_den_scan<R>), dim3(R * R / kWg, pb.units), dim3(kWg), 0, s, w.ScPart, w.Rchi, w.Rclo,
                           pb.t, pb.b / 256, pb.n / 256);
        PSF_LAUNCH_CHECK();
        constexpr int DC = 64;                              // value columns per re-layout workgroup
        const dim3 grid(R / 8, (unsigned)((size_t)pb.units * (pb.t - 1)), D / DC);
        hipLaunchKernelGGL((k_bwd_relayout<R, D, DC>), grid, dim3(kWg), 0, s, f.Zg, w.ZT);
        PSF_LAUNCH_CHECK();
        hipLaunchKernelGGL((k_bwd_relayout<R, D, DC>), grid, dim3(kWg), 0, s, w.Rg, w.RT);
        PSF_LAUNCH_CHECK();
    }
    if (tm) tm->mark();
    // in-block parts
    {
        const unsigned grid = (unsigned)(rows / (32 * NWL));
        if constexpr (R == D && P == 4) {
            if (ls) {
                hipLaunchKernelGGL((k_bwd_local_q<2, NWL, D>), dim3(grid), dim3(64 * NWL), 0, s, rq, w.KF, w.VF, w.K8,
                                   w.G_rm, w.Cc, w.dQacc, pb.n, pb.b);
                PSF_LAUNCH_CHECK();
            }
        }
        if (!ls) {
            hipLaunchKernelGGL((k_bwd_local_q<P, NWL, D>), dim3(grid), dim3(64 * NWL), 0, s, q, w.KF, w.VF, w.K8, w.G_rm,
                               w.Cc, w.dQacc, pb.n, pb.b);
            PSF_LAUNCH_CHECK();
        }
    }
    {
        // dV: the cross-block part first, the in-block kernel adds to it
        const unsigned gridc = (unsigned)(rows / (128 * TT)), grid = (unsigned)(rows / (32 * NWL));
        hipLaunchKernelGGL((k_bwd_dvc<R, D, TT>), dim3(gridc), dim3(kWg), 0, s, w.MK, w.Rg, w.dVc, pb.n, pb.b, pb.t);
        PSF_LAUNCH_CHECK();
        if constexpr (R == D && P == 4) {
            if (ls) {
                hipLaunchKernelGGL((k_bwd_local_k<2, NWL, D>), dim3(grid), dim3(64 * NWL), 0, s, w.QF, rk, v, w.Q8, w.GF,
                                   w.G8, w.Cc, w.dVc, w.dKacc, (bf16_t *)dV, pb.n, pb.b);
                PSF_LAUNCH_CHECK();
            }
        }
        if (!ls) {
            hipLaunchKernelGGL((k_bwd_local_k<P, NWL, D>), dim3(grid), dim3(64 * NWL), 0, s, w.QF, k, v, w.Q8, w.GF, w.G8,
                               w.Cc, w.dVc, w.dKacc, (bf16_t *)dV, pb.n, pb.b);
            PSF_LAUNCH_CHECK();
        }
    }
    if (tm) tm->mark();
    // cross-block parts of dm(q), dm(k), then through the sketch together with the in-block parts
    {
        const unsigned grid = (unsigned)(rows / (128 * TT));
        const int ph = pb.per_head ? 1 : 0;
        if constexpr (R == D && P == 4) {
            if (ls) {
                hipLaunchKernelGGL((k_bwd_dm<R, D, true, TT, true>), dim3(grid), dim3(kWg), 0, s, f.MQ, w.G_rm, w.Cc,
                                   w.ZT, f.Shi, f.Slo, q, f.Gt, (const bf16_t *)G, w.dQacc, (bf16_t *)dQ, pb.n, pb.b,
                                   pb.t, pb.heads, ph, pb.g_len);
                PSF_LAUNCH_CHECK();
                hipLaunchKernelGGL((k_bwd_dm<R, D, false, TT, true>), dim3(grid), dim3(kWg), 0, s, w.MK, v, w.Cc, w.RT,
                                   w.Rchi, w.Rclo, k, f.Gt, (const bf16_t *)G, w.dKacc, (bf16_t *)dK, pb.n, pb.b, pb.t,
                                   pb.heads, ph, pb.g_len);
                PSF_LAUNCH_CHECK();
            }
        }
        constexpr bool FUSED = D == 64 && P == 4;           // Algorithm 1's reverse inside k_bwd_dm
        if constexpr (FUSED) {
        if (pb.learned) {
            // dm as fp32 rows (in the buffer of the mirror-state octets, consumed by now), then
            // through the networks: one side after the other, the staging buffers serve both
            const int sets = pb.per_head ? pb.heads : 1;
            const unsigned grid_rows = (unsigned)(rows / 256);
            const int per_unit = learned_bwd_slices(pb), slice_rows = pb.n / per_unit;
            const unsigned grid_par = (unsigned)(pb.units * per_unit * 2 * (R / 4 / 4));
            hipLaunchKernelGGL((k_learned_bwd_prep<R>), dim3(4 * (R / 4), sets), dim3(kWg), 0, s, (const bf16_t *)G,
                               pb.g_len, w.LB);
            PSF_LAUNCH_CHECK();
            for (int side = 0; side < 2; ++side) {
                if (side == 0)
                    hipLaunchKernelGGL((k_bwd_dm<R, D, true, TT, false, true>), dim3(grid), dim3(kWg), 0, s, f.MQ, w.G_rm,
                                       w.Cc, w.ZT, f.Shi, f.Slo, q, nullptr, nullptr, nullptr, nullptr, pb.n, pb.b, pb.t,
                                       pb.heads, ph, pb.g_len, w.M8r);
                else
                    hipLaunchKernelGGL((k_bwd_dm<R, D, false, TT, false, true>), dim3(grid), dim3(kWg), 0, s, w.MK, v,
                                       w.Cc, w.RT, w.Rchi, w.Rclo, k, nullptr, nullptr, nullptr, nullptr, pb.n, pb.b, pb.t,
                                       pb.heads, ph, pb.g_len, w.M8r);
                PSF_LAUNCH_CHECK();
                const bf16_t *xr = side == 0 ? q : k;
                const float *base = side == 0 ? w.dQacc : w.dKacc;
                bf16_t *dx = (bf16_t *)(side == 0 ? dQ : dK);
                if (dG) {
                    hipLaunchKernelGGL((k_learned_bwd_rows<R, true>), dim3(grid_rows), dim3(512), 0, s, xr, w.M8r, base,
                                       f.LW, f.C1, f.LVp, w.LB, (const bf16_t *)G, pb.g_len, dx, w.sg, w.GB1, pb.n,
                                       pb.heads, ph);
                    PSF_LAUNCH_CHECK();
                    float *part = w.part + (size_t)side * pb.units * per_unit * pb.g_len;
                    hipLaunchKernelGGL((k_learned_bwd_params<R, 0>), dim3(grid_par), dim3(kWg), 0, s, w.sg,
                                       (const bf16_t *)G, pb.g_len, f.C1, w.GB1, part, pb.g_len, pb.n, slice_rows,
                                       pb.heads, ph);
                    PSF_LAUNCH_CHECK();
                    hipLaunchKernelGGL((k_learned_bwd_params<R, 1>), dim3(grid_par), dim3(kWg), 0, s, w.sg,
                                       (const bf16_t *)G, pb.g_len, f.C1, w.GB1, part, pb.g_len, pb.n, slice_rows,
                                       pb.heads, ph);
                    PSF_LAUNCH_CHECK();
                } else {
                    hipLaunchKernelGGL((k_learned_bwd_rows<R, false>), dim3(grid_rows), dim3(512), 0, s, xr, w.M8r, base,
                                       f.LW, f.C1, f.LVp, w.LB, (const bf16_t *)G, pb.g_len, dx, w.sg, w.GB1, pb.n,
                                       pb.heads, ph);
                    PSF_LAUNCH_CHECK();
                }
            }
            if (dG) {
                hipLaunchKernelGGL(k_learned_bwd_reduce, dim3((unsigned)((pb.g_len + kWg - 1) / kWg), sets), dim3(kWg), 0, s,
                                   w.part, dG, pb.g_len, pb.units, learned_bwd_slices(pb), pb.heads, ph);
                PSF_LAUNCH_CHECK();
            }
        } else if (!ls) {
            hipLaunchKernelGGL((k_bwd_dm<R, D, true, TT>), dim3(grid), dim3(kWg), 0, s, f.MQ, w.G_rm, w.Cc, w.ZT, f.Shi,
                               f.Slo, q, f.Gt, (const bf16_t *)G, w.dQacc, (bf16_t *)dQ, pb.n, pb.b, pb.t, pb.heads, ph,
                               pb.g_len);
            PSF_LAUNCH_CHECK();
            hipLaunchKernelGGL((k_bwd_dm<R, D, false, TT>), dim3(grid), dim3(kWg), 0, s, w.MK, v, w.Cc, w.RT, w.Rchi,
                               w.Rclo, k, f.Gt, (const bf16_t *)G, w.dKacc, (bf16_t *)dK, pb.n, pb.b, pb.t, pb.heads, ph,
                               pb.g_len);
            PSF_LAUNCH_CHECK();
        }
        } else {
            // d = 128 or degree 8: dm as fp32 rows (in the buffer of the mirror-state octets, consumed
            // by now), then Algorithm 1's reverse as a pass of its own, one side after the other
            for (int side = 0; side < 2; ++side) {
                if (side == 0)
                    hipLaunchKernelGGL((k_bwd_dm<R, D, true, TT, false, true>), dim3(grid), dim3(kWg), 0, s, f.MQ, w.G_rm,
                                       w.Cc, w.ZT, f.Shi, f.Slo, q, nullptr, nullptr, nullptr, nullptr, pb.n, pb.b, pb.t,
                                       pb.heads, ph, pb.g_len, w.M8r);
                else
                    hipLaunchKernelGGL((k_bwd_dm<R, D, false, TT, false, true>), dim3(grid), dim3(kWg), 0, s, w.MK, v,
                                       w.Cc, w.RT, w.Rchi, w.Rclo, k, nullptr, nullptr, nullptr, nullptr, pb.n, pb.b, pb.t,
                                       pb.heads, ph, pb.g_len, w.M8r);
                PSF_LAUNCH_CHECK();
                hipLaunchKernelGGL((k_bwd_sketch_rows<D, R, P>), dim3((unsigned)(rows / 128)), dim3(kWg), 0, s,
                                   side == 0 ? q : k, f.Gt, (const bf16_t *)G, w.M8r, side == 0 ? w.dQacc : w.dKacc,
                                   (bf16_t *)(side == 0 ? dQ : dK), pb.n, pb.heads, ph, pb.g_len);
                PSF_LAUNCH_CHECK();
            }
        }
    }
    if (tm) tm->mark();
    return PSF_OK;
}
