// Backward pass through the learned sketches (Algorithm 2, degree 4, networks of Appendix D) on
// MFMA: bf16 storage, d = 64, r in {32, 64}.  Included inside the anonymous namespace of
// psf_mfma.hip before psf_mfma_bwd.inl, whose kernels leave dL/dm(Q), dL/dm(K) as fp32 rows and
// whose host code launches these.
//
// m = sqrt(r) tanh(f1(x) f2(x) / sqrt(r)); with z = f1 f2:  dz = dm (1 - tanh^2),  df1 = dz f2,
// df2 = dz f1.  One network (x^ = normalised row, u1 = g1 x^ + b1, a1 = u1 W1, h1 = gelu(a1),
// h^ = normalised h1, u2 = g2 h^ + b2, a2 = u2 W2, a3 = a2 W3, h3 = gelu(a3), f = h3 W4), reverse:
//     dW4 = sum h3 (x) df        dh3 = W4 df         da3 = dh3 gelu'(a3)
//     dW3 = sum a2 (x) da3       da2 = W3 da3
//     dW2 = sum u2 (x) da2       du2 = W2 da2        dg2 = sum du2 h^     db2 = sum du2
//     dh1 = (g2 du2 - m1 - h^ m2) / sigma2,  m1 = mean(g2 du2) = <s2, da2> / 8r  (s2 = column sums of g2 . W2),
//                                           m2 = mean(g2 du2 h^) = <da2, a2 - b2 W2> / 8r
//     da1 = dh1 gelu'(a1)
//     dW1 = sum u1 (x) da1       du1 = W1 da1        dg1 = sum du1 x^     db1 = sum du1
//     dx  = (g1 du1 - mean(g1 du1) - x^ mean(g1 du1 x^)) / sigma1
// (sums over the rows that share the parameter set).  Both layer-normalisation means of the
// hidden layer are functions of r-wide vectors, so no pass over the 8r hidden units is needed
// before their gradients can be formed.
//
// Two kernels per side (query rows, key rows):
//   k_learned_bwd_rows    workgroup = 256 rows, lane = row ("[feature][row]" accumulators as in
//                         k_learned_sketch): both networks forward, the node, then per network the
//                         chain df -> da2 -> du1 -> dx with the hidden units walked in chunks of 32
//                         (pre-activations recomputed per chunk); writes dX = bf16(direct term + dx),
//                         the sums for dg1 / db1 per workgroup, and, for the parameter kernel, the
//                         r-wide vectors of every row (x^, a2, df, da2 as bf16, once as row
//                         operands and once as transposed operands of the parameter kernel's
//                         MFMAs, both in the order its lanes load them: see LbStage; mean and
//                         1/sigma of h1, m1, m2).
//   k_learned_bwd_params  workgroup = 4 waves = 4 hidden chunks of one network for a slice of the rows
//                         of one unit, lane = hidden unit: recomputes a1 (or a3) of its 32 hidden units
//                         with the operand roles swapped ("[row][hidden]" accumulators), forms h1, h^,
//                         da1 (h3, da3) there, and contracts over the rows on MFMA with the staged
//                         tiles as the other operand; the sums over the slice stay in accumulators and
//                         are written once, in the layout of the parameter blob.
//   k_learned_bwd_reduce  adds the per-slice parts in a fixed order (no atomics: a repeated call
//                         returns the same bits).

constexpr int kLbSlot = 16384;          // backward weight slot of one hidden chunk: three parts of 4 KB + padding
constexpr int kLbRing = 4;

__device__ __forceinline__ void gelu_and_slope(float x, float &y, float &dy)
{
    // gelu(x) = x s, s = 1 / (1 + exp(-2u)), 2u = x (1.5957691 + 0.0713548 x^2) (tanh form);
    // gelu'(x) = s + x s (1 - s) d(2u)/dx.  Finite for |x| < 1e19.
    const float x2 = x * x;
    const float e = __builtin_amdgcn_exp2f(x * (2.3022082f + 0.10294324f * x2));
    const float rc = __builtin_amdgcn_rcpf(1.0f + e);         // 1 - s
    const float s = 1.0f - rc;
    y = x * s;
    dy = s + x * rc * s * (1.5957691f + 0.2140645f * x2);
}

// Slot (net, phase, chunk) of the backward weight stream of one parameter set; grid (4 * NCH, sets).
// Fragment (blk, i, h, e) sits at ((blk * 32 + i) * 2 + h) * 8 + e of its part; perm = 8 (e / 4) + 4 h + e % 4
// is the accumulator row order inside a k-step of 16, feat = 32 (blk / 2) + 16 (blk % 2) + perm,
// hidp = 32 ch + 16 (blk % 2) + perm.
//   phase 0 (layers 3, 4):  part 0  W3[feat][32 ch + i]            (a3 again, as in the forward stream)
//                           part 1  W4[32 ch + i][feat]            (dh3 = W4 df)
//                           part 2  W3[32 (blk / 2) + i][hidp]     (da2 += W3 da3)
//   phase 1 (layers 1, 2):  part 0  g1[k] W1[k][32 ch + i], k = 16 blk + 8 h + e   (a1 again)
//                           part 1  g2[hid] W2[hid][feat], hid = 32 ch + i         (g2 du2)
//                           part 2  W1[32 (blk / 2) + i][hidp]                     (du1 += W1 da1)
template <int R>
__global__ __launch_bounds__(kWg) void k_learned_bwd_prep(const bf16_t *__restrict__ P, size_t p_len,
                                                          bf16_t *__restrict__ LB)
{
    using Net = LearnedNet<R, 64>;
    constexpr int NCH = Net::NCH, HID = Net::HID, OT = R / 32, RS = R / 16;
    const int q = blockIdx.x, set = blockIdx.y, tid = threadIdx.x;
    const int net = q / (2 * NCH), phase = (q / NCH) % 2, ch = q % NCH;
    const Net nt(P + (size_t)set * p_len + Net::offset_of(net, 4), 64);
    bf16_t *slot = LB + ((size_t)set * 4 * NCH + q) * (kLbSlot / 2);
    for (int idx = tid; idx < kLbSlot / 2; idx += kWg) {
        const int part = idx / 2048, r2 = idx % 2048;
        const int blk = r2 / 512, i = (r2 % 512) / 16, h = (r2 / 8) % 2, e = r2 % 8;
        const int perm = 8 * (e / 4) + 4 * h + e % 4;
        const int feat = 32 * (blk / 2) + 16 * (blk % 2) + perm, hidp = 32 * ch + 16 * (blk % 2) + perm;
        const int hid = 32 * ch + i;
        float v = 0.f;
        if (phase == 0) {
            if (part == 0 && blk < RS) v = bf16_to_f32(nt.W3[(size_t)feat * HID + hid]);
            if (part == 1 && blk < RS) v = bf16_to_f32(nt.W4[(size_t)hid * R + feat]);
            if (part == 2 && blk < 2 * OT) v = bf16_to_f32(nt.W3[(size_t)(32 * (blk / 2) + i) * HID + hidp]);
        } else {
            if (part == 0) {
                const int k = 16 * blk + 8 * h + e;
                v = bf16_to_f32(nt.g1[k]) * bf16_to_f32(nt.W1[(size_t)k * HID + hid]);
            }
            if (part == 1 && blk < RS) v = bf16_to_f32(nt.g2[hid]) * bf16_to_f32(nt.W2[(size_t)hid * R + feat]);
            if (part == 2) v = bf16_to_f32(nt.W1[(size_t)(32 * (blk / 2) + i) * HID + hidp]);
        }
        // part 0 meets activations (the forward operand type), parts 1 and 2 gradients (bf16: their range
        // is the caller's loss scale); part 3 is padding
        slot[idx] = part == 0 ? LsOp<kLsHalf>::bits(v) : f32_to_bf16(v);
    }
}

// What k_learned_bwd_rows leaves for k_learned_bwd_params, per side.  rows = units * n.
//   XnR [rows/32][64/16][2][32][8]      normalised rows x^ (bf16): tile, k-step, half, row, 8 features
//                                       16 step + 8 half + e -- what a lane (row, half) feeds an MFMA as a row operand
//   XnT [rows/32][64/32][2][2][32][8]   the same transposed: tile, feature tile, k-step s2, half, feature, 8 rows
//                                       16 s2 + 8 (e / 4) + 4 half + e % 4 -- the operand of a lane (feature, half)
//   (either way a wave's load instruction takes 1 KB in one piece: with plain row-major arrays every
//   lane touched a cache line of its own and the parameter kernel was bound by the vector L1's line rate)
//   per network (stride rows * R): A2R / A2T (a2), DOR / DOT (df), DAR / DAT (da2), laid out alike with R features
//   ST  [net][4][rows] fp32   mean of h1, 1 / sigma2, m1, m2
struct LbStage {
    bf16_t *XnR, *XnT, *A2R, *A2T, *DOR, *DOT, *DAR, *DAT;
    float *ST;
    size_t rows;
};

// dM: dL/dm of the rows as fp32 [rows][R]; dXacc: the direct term of the exact in-block weights
// (fp32 [rows][64]); LW, C1, LVp: the forward weight stream of k_learned_prep; LB: the backward
// stream; P: the parameter blobs (for g1).  GB1: [workgroup][net][2][64] fp32, the workgroup's sums
// for dg1 and db1.  STAGE = false: row gradient only (parameters as constants).
template <int R, bool STAGE>
__global__ __launch_bounds__(512, 1) void k_learned_bwd_rows(const bf16_t *__restrict__ X, const float *__restrict__ dM,
                                                            const float *__restrict__ dXacc,
                                                            const bf16_t *__restrict__ LW, const float *__restrict__ C1,
                                                            const float *__restrict__ LVp,
                                                            const bf16_t *__restrict__ LB, const bf16_t *__restrict__ P,
                                                            size_t p_len, bf16_t *__restrict__ dX, LbStage sg,
                                                            float *__restrict__ GB1, int n, int heads, int per_head)
{
    using Net = LearnedNet<R, 64>;
    constexpr int NCH = Net::NCH, HID = Net::HID, D = 64, OT = R / 32, KS = D / 16, RS = R / 16, DT = D / 32;
    constexpr int FSLOT = kLsSlotBytes, FPART1 = FSLOT / 2, NTHR = 512, NETS = 2;
    constexpr int QN = 2 * NETS * NCH;                     // slots of either weight stream
    constexpr int FDMA = FSLOT / 16 / NTHR, BDMA = kLbSlot / 16 / NTHR;
    static_assert(FDMA == 1 && BDMA == 2, "copies per thread and slot");
    __shared__ __attribute__((aligned(16))) unsigned char ring[kLbRing * kLbSlot];
    __shared__ __attribute__((aligned(16))) float c1s[NETS * NCH * 32];
    __shared__ __attribute__((aligned(16))) float lv[NETS * 2 * R];
    __shared__ float red[8][NETS][2][D];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 31, h = lane >> 5;
    const size_t row0 = (size_t)blockIdx.x * 256;
    const size_t row = row0 + wave * 32 + x;
    const int set = per_head ? (int)((row0 / n) % heads) : 0;
    const unsigned char *fstream = (const unsigned char *)(LW + (size_t)set * QN * (FSLOT / 2));
    const unsigned char *bstream = (const unsigned char *)(LB + (size_t)set * QN * (kLbSlot / 2));
    const uint32_t ring0 = lds_address(ring);
    auto stage_f = [&](int q) {
        const int qc = min(q, QN - 1);                     // clamped: keeps the copy count uniform
        dma16_sbase(fstream + (size_t)qc * FSLOT, (uint32_t)tid * 16, ring0 + (q % kLbRing) * FSLOT + wave * 1024);
    };
    auto stage_b = [&](int q) {
        const int qc = min(q, QN - 1);
#pragma unroll
        for (int c = 0; c < BDMA; ++c)
            dma16_sbase(bstream + (size_t)qc * kLbSlot + c * (NTHR * 16), (uint32_t)tid * 16,
                        ring0 + (q % kLbRing) * kLbSlot + c * (NTHR * 16) + wave * 1024);
    };
#pragma unroll
    for (int q = 0; q < kLbRing - 1; ++q) stage_f(q);
    for (int idx = tid; idx < NETS * NCH * 32; idx += NTHR) c1s[idx] = C1[(size_t)set * NETS * NCH * 32 + idx];
    for (int idx = tid; idx < NETS * 2 * R; idx += NTHR) { // s2, c2: sum of the per-chunk parts
        const int net = idx / (2 * R), rest = idx % (2 * R);
        const float *src = LVp + ((size_t)set * NETS + net) * NCH * 2 * R + rest;
        float acc = 0.f;
        for (int ch = 0; ch < NCH; ++ch) acc += src[(size_t)ch * 2 * R];
        lv[idx] = acc;
    }

    // Products of weights with activations run in the forward kernel's operand type, products
    // with gradients in bf16.
    using OpA = LsOp<kLsHalf>;
    typedef typename OpA::v8 a8;
    // ---- the row, normalised: B operands of the first layer ----
    a8 xfr[KS];
    float mean1, inv1;
    {
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
        mean1 = sum * (1.0f / D);
        inv1 = rsqrtf(fmaxf(sq * (1.0f / D) - mean1 * mean1, 0.f) + 1e-6f);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) xfr[s][e] = (typename OpA::elem)((xv[s][e] - mean1) * inv1);
    }

    // ---- both networks forward (k_learned_sketch's arithmetic) ----
    a8 h2f[NETS][RS];                                       // a2 as the B operand of the third layer
    bf16x8 a2b[STAGE ? NETS : 1][RS];                       // the same as bf16, for the parameter kernel
    f32x16 fo[NETS][OT];                                    // network outputs
    float mean2[NETS], inv2[NETS];
    int q = 0;
#pragma unroll
    for (int net = 0; net < NETS; ++net) {
        f32x16 acc2[OT];
        float sh = 0.f, sqh = 0.f;
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) acc2[ot] = f32x16{0};
#pragma unroll 1
        for (int ch = 0; ch < NCH; ++ch, ++q) {
            wait_vmem_le<(kLbRing - 2) * FDMA>();
            __syncthreads();                               // slot q has landed for everybody; slot q-1 is free
            stage_f(q + kLbRing - 1);
            const unsigned char *sl = ring + (q % kLbRing) * FSLOT;
            f32x16 acc;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 c = *(const f32x4 *)&c1s[(net * NCH + ch) * 32 + 8 * g4 + 4 * h];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) acc[4 * g4 + j2] = c[j2];
            }
#pragma unroll
            for (int s = 0; s < KS; ++s) acc = OpA::mfma(*(const a8 *)(sl + ((s * 32 + x) * 2 + h) * 16), xfr[s], acc);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float hv = gelu_poly(acc[v]);
                sh += hv;
                sqh += hv * hv;
                acc[v] = hv;
            }
            const a8 hf0 = ls_cvt_from16<OpA>(acc, 0), hf1 = ls_cvt_from16<OpA>(acc, 8);
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
                acc2[ot] = OpA::mfma(*(const a8 *)(sl + FPART1 + (((ot * 2 + 0) * 32 + x) * 2 + h) * 16), hf0, acc2[ot]);
                acc2[ot] = OpA::mfma(*(const a8 *)(sl + FPART1 + (((ot * 2 + 1) * 32 + x) * 2 + h) * 16), hf1, acc2[ot]);
            }
        }
        {
            const float s_all = sh + __shfl_xor(sh, 32), q_all = sqh + __shfl_xor(sqh, 32);
            mean2[net] = s_all * (1.0f / HID);
            inv2[net] = rsqrtf(fmaxf(q_all * (1.0f / HID) - mean2[net] * mean2[net], 0.f) + 1e-6f);
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const f32x4 s2 = *(const f32x4 *)&lv[(net * 2 + 0) * R + 32 * ot + 8 * g4 + 4 * h];
                    const f32x4 c2 = *(const f32x4 *)&lv[(net * 2 + 1) * R + 32 * ot + 8 * g4 + 4 * h];
#pragma unroll
                    for (int j2 = 0; j2 < 4; ++j2)
                        acc2[ot][4 * g4 + j2] = (acc2[ot][4 * g4 + j2] - mean2[net] * s2[j2]) * inv2[net] + c2[j2];
                }
                h2f[net][2 * ot] = ls_cvt_from16<OpA>(acc2[ot], 0);
                h2f[net][2 * ot + 1] = ls_cvt_from16<OpA>(acc2[ot], 8);
                if constexpr (STAGE) {
                    a2b[net][2 * ot] = cvt8_from16(acc2[ot], 0);
                    a2b[net][2 * ot + 1] = cvt8_from16(acc2[ot], 8);
                }
            }
        }
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) fo[net][ot] = f32x16{0};
#pragma unroll 1
        for (int ch = 0; ch < NCH; ++ch, ++q) {
            wait_vmem_le<(kLbRing - 2) * FDMA>();
            __syncthreads();
            stage_f(q + kLbRing - 1);
            const unsigned char *sl = ring + (q % kLbRing) * FSLOT;
            f32x16 acc = {0};
#pragma unroll
            for (int t = 0; t < RS; ++t) acc = OpA::mfma(*(const a8 *)(sl + ((t * 32 + x) * 2 + h) * 16), h2f[net][t], acc);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = gelu_poly(acc[v]);
            const a8 hf0 = ls_cvt_from16<OpA>(acc, 0), hf1 = ls_cvt_from16<OpA>(acc, 8);
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
                fo[net][ot] = OpA::mfma(*(const a8 *)(sl + FPART1 + (((ot * 2 + 0) * 32 + x) * 2 + h) * 16), hf0, fo[net][ot]);
                fo[net][ot] = OpA::mfma(*(const a8 *)(sl + FPART1 + (((ot * 2 + 1) * 32 + x) * 2 + h) * 16), hf1, fo[net][ot]);
            }
        }
    }
    wait_vmem_le<0>();                                     // drain the clamped copies of the forward stream
    __syncthreads();                                       // every wave is done with the forward slots
#pragma unroll
    for (int qq = 0; qq < kLbRing - 1; ++qq) stage_b(qq);

    // ---- the node: df1 = dz f2, df2 = dz f1, dz = dm (1 - tanh^2(f1 f2 / sqrt r)) ----
    // register v of tile ot: feature 32 ot + 8 (v / 4) + 4 h + v % 4
    const size_t tile = row0 / 32 + wave;                  // tile of 32 rows in the transposed copies
    bf16x8 dof[NETS][RS];
    {
        const float isr = 1.0f / sqrtf((float)R);
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
            f32x16 d0, d1;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 dm4 = *(const f32x4 *)&dM[row * R + 32 * ot + 8 * g4 + 4 * h];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) {
                    const int v = 4 * g4 + j2;
                    const float t = tanh_fast(fo[0][ot][v] * fo[1][ot][v] * isr);
                    const float dz = dm4[j2] * (1.0f - t * t);
                    d0[v] = dz * fo[1][ot][v];
                    d1[v] = dz * fo[0][ot][v];
                }
            }
            dof[0][2 * ot] = cvt8_from16(d0, 0);
            dof[0][2 * ot + 1] = cvt8_from16(d0, 8);
            dof[1][2 * ot] = cvt8_from16(d1, 0);
            dof[1][2 * ot + 1] = cvt8_from16(d1, 8);
        }
    }
    // bf16 fragments (k-step t, entries e: feature 16 t + 8 (e / 4) + 4 h + e % 4) go out twice, both in
    // the order the parameter kernel's lanes load them, 1 KB per load instruction in one piece:
    //   rows   [tile][k-step][half][row 0..31][8]       : feature 16 step + 8 half + e of the row
    //   tiles  [tile][feature / 32][k-step s2][half][feature % 32][8] : row 16 s2 + 8 (e / 4) + 4 half + e % 4
    const int tslot = ((x >> 4) * 2 + ((x >> 2) & 1)) * 256 + 4 * ((x >> 3) & 1) + (x & 3);
    auto stage_vec = [&](const bf16x8 (&f)[RS], bf16_t *rows_out, bf16_t *tile_out) {
#pragma unroll
        for (int t = 0; t < RS; ++t)
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2) {
                const bf16x4 p4 = {f[t][4 * g2], f[t][4 * g2 + 1], f[t][4 * g2 + 2], f[t][4 * g2 + 3]};
                *(bf16x4 *)&rows_out[((tile * RS + t) * 2 + g2) * 256 + x * 8 + 4 * h] = p4;
                // (the 16-bit pieces are cut from the 32-bit words: a bit cast of single vector elements
                // stored the first element of every group of four for all four)
                const uint2 bits = __builtin_bit_cast(uint2, p4);
                bf16_t *col = tile_out + (tile * OT + t / 2) * 1024 + tslot + (16 * (t % 2) + 8 * g2 + 4 * h) * 8;
                col[0] = (bf16_t)(bits.x & 0xffffu);
                col[8] = (bf16_t)(bits.x >> 16);
                col[16] = (bf16_t)(bits.y & 0xffffu);
                col[24] = (bf16_t)(bits.y >> 16);
            }
    };
    if constexpr (STAGE) {
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            bf16x8 xb;
#pragma unroll
            for (int e = 0; e < 8; ++e) xb[e] = (__bf16)(float)xfr[s][e];
            *(bf16x8 *)&sg.XnR[((tile * KS + s) * 2 + h) * 256 + x * 8] = xb;
            const uint4 bits = __builtin_bit_cast(uint4, xb);
            const uint32_t wd[4] = {bits.x, bits.y, bits.z, bits.w};
            bf16_t *col = sg.XnT + (tile * DT + s / 2) * 1024 + tslot + (16 * (s % 2) + 8 * h) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) col[8 * e] = (bf16_t)((wd[e / 2] >> (16 * (e % 2))) & 0xffffu);
        }
#pragma unroll
        for (int net = 0; net < NETS; ++net) {
            stage_vec(a2b[net], sg.A2R + (size_t)net * sg.rows * R, sg.A2T + (size_t)net * sg.rows * R);
            stage_vec(dof[net], sg.DOR + (size_t)net * sg.rows * R, sg.DOT + (size_t)net * sg.rows * R);
            if (h == 0) {
                sg.ST[((size_t)net * 4 + 0) * sg.rows + row] = mean2[net];
                sg.ST[((size_t)net * 4 + 1) * sg.rows + row] = inv2[net];
            }
        }
    }

    // ---- reverse, network by network ----
    f32x16 dxs[DT];                                         // dx, feature 32 dt + 8 (v / 4) + 4 h + v % 4
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) dxs[dt] = f32x16{0};
    f32x16 xh[DT];                                          // x^ in that order
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const bf16x4 raw = *(const bf16x4 *)&X[row * D + 32 * dt + 8 * g4 + 4 * h];
#pragma unroll
            for (int j2 = 0; j2 < 4; ++j2) xh[dt][4 * g4 + j2] = ((float)raw[j2] - mean1) * inv1;
        }
    q = 0;
#pragma unroll
    for (int net = 0; net < NETS; ++net) {
        // layers 4 and 3
        f32x16 da2[OT];
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) da2[ot] = f32x16{0};
#pragma unroll 1
        for (int ch = 0; ch < NCH; ++ch, ++q) {
            wait_vmem_le<(kLbRing - 2) * BDMA>();
            __syncthreads();
            stage_b(q + kLbRing - 1);
            const unsigned char *sl = ring + (q % kLbRing) * kLbSlot;
            f32x16 a3 = {0}, dh3 = {0};
#pragma unroll
            for (int t = 0; t < RS; ++t) {
                a3 = OpA::mfma(*(const a8 *)(sl + ((t * 32 + x) * 2 + h) * 16), h2f[net][t], a3);
                dh3 = mfma32(*(const bf16x8 *)(sl + 4096 + ((t * 32 + x) * 2 + h) * 16), dof[net][t], dh3);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float y, dy;
                gelu_and_slope(a3[v], y, dy);
                dh3[v] *= dy;
            }
            const bf16x8 df0 = cvt8_from16(dh3, 0), df1 = cvt8_from16(dh3, 8);
#pragma unroll
            for (int ot = 0; ot < OT; ++ot) {
                da2[ot] = mfma32(*(const bf16x8 *)(sl + 8192 + (((ot * 2 + 0) * 32 + x) * 2 + h) * 16), df0, da2[ot]);
                da2[ot] = mfma32(*(const bf16x8 *)(sl + 8192 + (((ot * 2 + 1) * 32 + x) * 2 + h) * 16), df1, da2[ot]);
            }
        }
        // the two means of the hidden layer normalisation's reverse
        float m1 = 0.f, m2 = 0.f;
        bf16x8 daf[RS];
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 s2 = *(const f32x4 *)&lv[(net * 2 + 0) * R + 32 * ot + 8 * g4 + 4 * h];
                const f32x4 c2 = *(const f32x4 *)&lv[(net * 2 + 1) * R + 32 * ot + 8 * g4 + 4 * h];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) {
                    const int v = 4 * g4 + j2;
                    const float a2v = (float)h2f[net][2 * ot + v / 8][v % 8];
                    m1 += s2[j2] * da2[ot][v];
                    m2 += da2[ot][v] * (a2v - c2[j2]);
                }
            }
            daf[2 * ot] = cvt8_from16(da2[ot], 0);
            daf[2 * ot + 1] = cvt8_from16(da2[ot], 8);
        }
        m1 = (m1 + __shfl_xor(m1, 32)) * (1.0f / HID);
        m2 = (m2 + __shfl_xor(m2, 32)) * (1.0f / HID);
        if constexpr (STAGE) {
            stage_vec(daf, sg.DAR + (size_t)net * sg.rows * R, sg.DAT + (size_t)net * sg.rows * R);
            if (h == 0) {
                sg.ST[((size_t)net * 4 + 2) * sg.rows + row] = m1;
                sg.ST[((size_t)net * 4 + 3) * sg.rows + row] = m2;
            }
        }
        // layers 2 and 1
        f32x16 du1[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) du1[dt] = f32x16{0};
        const float mu = mean2[net], iv = inv2[net];
#pragma unroll 1
        for (int ch = 0; ch < NCH; ++ch, ++q) {
            wait_vmem_le<(kLbRing - 2) * BDMA>();
            __syncthreads();
            stage_b(q + kLbRing - 1);
            const unsigned char *sl = ring + (q % kLbRing) * kLbSlot;
            f32x16 a1, dhh = {0};
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 c = *(const f32x4 *)&c1s[(net * NCH + ch) * 32 + 8 * g4 + 4 * h];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) a1[4 * g4 + j2] = c[j2];
            }
#pragma unroll
            for (int s = 0; s < KS; ++s) a1 = OpA::mfma(*(const a8 *)(sl + ((s * 32 + x) * 2 + h) * 16), xfr[s], a1);
#pragma unroll
            for (int t = 0; t < RS; ++t) dhh = mfma32(*(const bf16x8 *)(sl + 4096 + ((t * 32 + x) * 2 + h) * 16), daf[t], dhh);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float y, dy;
                gelu_and_slope(a1[v], y, dy);
                const float hh = (y - mu) * iv;
                dhh[v] = iv * (dhh[v] - m1 - hh * m2) * dy;
            }
            const bf16x8 df0 = cvt8_from16(dhh, 0), df1 = cvt8_from16(dhh, 8);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                du1[dt] = mfma32(*(const bf16x8 *)(sl + 8192 + (((dt * 2 + 0) * 32 + x) * 2 + h) * 16), df0, du1[dt]);
                du1[dt] = mfma32(*(const bf16x8 *)(sl + 8192 + (((dt * 2 + 1) * 32 + x) * 2 + h) * 16), df1, du1[dt]);
            }
        }
        // first layer normalisation; sums over the wave's 32 rows for dg1, db1
        const bf16_t *g1 = P + (size_t)set * p_len + Net::offset_of(net, 4);
        float mA = 0.f, mB = 0.f;
        f32x16 dxh[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const bf16x4 gg = *(const bf16x4 *)&g1[32 * dt + 8 * g4 + 4 * h];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) {
                    const int v = 4 * g4 + j2;
                    const float d = du1[dt][v];
                    dxh[dt][v] = (float)gg[j2] * d;
                    mA += dxh[dt][v];
                    mB += dxh[dt][v] * xh[dt][v];
                    if constexpr (STAGE) {
                        float sg1 = d * xh[dt][v], sb1 = d;
#pragma unroll
                        for (int m = 1; m < 32; m *= 2) {
                            sg1 += __shfl_xor(sg1, m);
                            sb1 += __shfl_xor(sb1, m);
                        }
                        if (x == 0) {
                            red[wave][net][0][32 * dt + 8 * g4 + 4 * h + j2] = sg1;
                            red[wave][net][1][32 * dt + 8 * g4 + 4 * h + j2] = sb1;
                        }
                    }
                }
            }
        mA = (mA + __shfl_xor(mA, 32)) * (1.0f / D);
        mB = (mB + __shfl_xor(mB, 32)) * (1.0f / D);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) dxs[dt][v] += inv1 * (dxh[dt][v] - mA - xh[dt][v] * mB);
    }
    wait_vmem_le<0>();                                     // drain the clamped copies

#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const size_t off = row * D + 32 * dt + 8 * g4 + 4 * h;
            f32x4 o4 = {dxs[dt][4 * g4], dxs[dt][4 * g4 + 1], dxs[dt][4 * g4 + 2], dxs[dt][4 * g4 + 3]};
            const f32x4 base = *(const f32x4 *)&dXacc[off];
#pragma unroll
            for (int j2 = 0; j2 < 4; ++j2) o4[j2] += base[j2];
            *(bf16x4 *)&dX[off] = cvt4(o4);
        }
    if constexpr (STAGE) {
        __syncthreads();
        if (tid < NETS * 2 * D) {
            float sum = 0.f;
#pragma unroll
            for (int wv = 0; wv < 8; ++wv) sum += (&red[wv][0][0][0])[tid];
            GB1[(size_t)blockIdx.x * NETS * 2 * D + tid] = sum;
        }
    }
}

// Parameter sums over one slice (slice_rows consecutive rows of one unit, a multiple of 256) for
// the 4 hidden chunks (one per wave) of group cg of network net; lane = hidden unit 32 ch + x.
// HALF 0: layers 1 and 2 (W1, g2, b2, W2; its first workgroup of a network also sums g1 / b1 from
// the row kernel's workgroup sums GB1), HALF 1: layers 3 and 4 (W3, W4): two sets of
// accumulators that do not share a register budget.  part: fp32 copy of the parameter blob per
// slice, every entry of networks 0 and 1 written exactly once over the launch.
template <int R, int HALF>
__global__ __launch_bounds__(kWg, 2) void k_learned_bwd_params(LbStage sg, const bf16_t *__restrict__ P, size_t p_len,
                                                              const float *__restrict__ C1,
                                                              const float *__restrict__ GB1, float *__restrict__ part,
                                                              size_t blob_len, int n, int slice_rows, int heads,
                                                              int per_head)
{
    using Net = LearnedNet<R, 64>;
    constexpr int NCH = Net::NCH, HID = Net::HID, D = 64, OT = R / 32, KS = D / 16, RS = R / 16, DT = D / 32;
    constexpr int CG = NCH / 4, JOBS = 2 * CG;             // workgroups per slice
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 31, h = lane >> 5;
    // the workgroups of one slice read the same staged rows: keep them on one XCD (one L2)
    int wg = blockIdx.x;
    const int total = gridDim.x;
    if ((total / JOBS) % 8 == 0) {
        const int xcd = wg & 7, idx = wg >> 3;
        wg = ((idx / JOBS) * 8 + xcd) * JOBS + idx % JOBS;
    }
    const int slice = wg / JOBS, net = (wg % JOBS) / CG, cg = wg % CG;
    const int per_unit = n / slice_rows;
    const int u = slice / per_unit;
    const size_t first = (size_t)u * n + (size_t)(slice % per_unit) * slice_rows;
    const int ch = cg * 4 + wave, hid = 32 * ch + x;
    const int set = per_head ? u % heads : 0;
    const Net nt(P + (size_t)set * p_len + Net::offset_of(net, 4), 64);

    // HALF 0: the four statistics of a tile's 32 rows, per wave (every lane needs those of the
    // rows of its accumulator registers, the same for 32 lanes: as global loads those cost a
    // cache access per lane, through workgroup memory one broadcast read)
    __shared__ __attribute__((aligned(16))) float stl[HALF == 0 ? 4 : 1][128];
    // this chunk's weights as B operands (lane = hidden unit, 8 consecutive contraction indices)
    bf16x8 wa[HALF == 0 ? KS : RS], wb[RS];                // HALF 0: g1 . W1, W2;  HALF 1: W3, W4
    if constexpr (HALF == 0) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = 16 * s + 8 * h + e;
                wa[s][e] = (__bf16)(bf16_to_f32(nt.g1[k]) * bf16_to_f32(nt.W1[(size_t)k * HID + hid]));
            }
    }
#pragma unroll
    for (int t = 0; t < RS; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = 16 * t + 8 * h + e;
            if constexpr (HALF == 0) {
                wb[t][e] = __builtin_bit_cast(__bf16, nt.W2[(size_t)hid * R + k]);
            } else {
                wa[t][e] = __builtin_bit_cast(__bf16, nt.W3[(size_t)k * HID + hid]);
                wb[t][e] = __builtin_bit_cast(__bf16, nt.W4[(size_t)hid * R + k]);
            }
        }
    const float c1 = C1[(((size_t)set * 2 + net) * NCH + ch) * 32 + x];
    const float g2h = bf16_to_f32(nt.g2[hid]);

    // HALF 0: accA = dW1 (DT tiles), accB = dW2;  HALF 1: accA = dW3, accB = dW4
    constexpr int NA = HALF == 0 ? DT : OT;
    f32x16 accA[NA], accB[OT];
#pragma unroll
    for (int i = 0; i < NA; ++i) accA[i] = f32x16{0};
#pragma unroll
    for (int ot = 0; ot < OT; ++ot) accB[ot] = f32x16{0};
    float sg2 = 0.f, sb2 = 0.f, sda1 = 0.f, sda2[OT];
#pragma unroll
    for (int ot = 0; ot < OT; ++ot) sda2[ot] = 0.f;

    const bf16_t *A2R = sg.A2R + (size_t)net * sg.rows * R, *A2T = sg.A2T + (size_t)net * sg.rows * R;
    const bf16_t *DOR = sg.DOR + (size_t)net * sg.rows * R, *DOT = sg.DOT + (size_t)net * sg.rows * R;
    const bf16_t *DAR = sg.DAR + (size_t)net * sg.rows * R, *DAT = sg.DAT + (size_t)net * sg.rows * R;
    const float *ST = sg.ST + (size_t)net * 4 * sg.rows;
    // 8 rows of a transposed tile in the accumulator order of k-step s2 (16 s2 + 4 h + {0..3}, + 8) of
    // feature 32 ft + x: one 16-byte piece per lane, the wave's 1 KB in one run
    auto frag_t = [&](const bf16_t *T, size_t tile, int tiles_wide, int ft, int s2) {
        return *(const bf16x8 *)&T[((tile * tiles_wide + ft) * 2 + s2) * 512 + (h * 32 + x) * 8];
    };
    auto frag_r = [&](const bf16_t *Rw, size_t tile, int steps, int s) {
        return *(const bf16x8 *)&Rw[((tile * steps + s) * 2 + h) * 256 + x * 8];
    };

    // operands of one tile of 32 rows: row fragments (lane = row) of two staged vectors and the
    // transposed tiles (lane = feature) of two; the next tile's are loaded under the current one's arithmetic
    struct Tile {
        bf16x8 ra[HALF == 0 ? KS : RS], rb[RS];            // HALF 0: x^, da2;  HALF 1: a2, df
        bf16x8 ta[NA][2], tb[OT][2];                       // HALF 0: x^ tiles, da2 tiles;  HALF 1: a2 tiles, df tiles
        float st[2];                                       // HALF 0: statistics h and 2 + h of row x
    };
    // (HALF 0 is short of registers: there only the row fragments, which the tile's first products
    // wait for, come a tile ahead; the transposed tiles are asked for at the top of their own tile
    // and used at its end)
    auto load_tile = [&](int tl, Tile &o, bool rows_part, bool tiles_part) {
        const size_t tile = (first + 32 * (size_t)tl) / 32;
        if constexpr (HALF == 0) {
            if (rows_part) {
#pragma unroll
                for (int s = 0; s < KS; ++s) o.ra[s] = frag_r(sg.XnR, tile, KS, s);
#pragma unroll
                for (int t = 0; t < RS; ++t) o.rb[t] = frag_r(DAR, tile, RS, t);
                o.st[0] = ST[(size_t)h * sg.rows + tile * 32 + x];
                o.st[1] = ST[(size_t)(2 + h) * sg.rows + tile * 32 + x];
            }
            if (tiles_part)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) o.ta[dt][s2] = frag_t(sg.XnT, tile, DT, dt, s2);
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) o.tb[ot][s2] = frag_t(DAT, tile, OT, ot, s2);
            }
        } else {
#pragma unroll
            for (int t = 0; t < RS; ++t) {
                o.ra[t] = frag_r(A2R, tile, RS, t);
                o.rb[t] = frag_r(DOR, tile, RS, t);
            }
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) {
                    o.ta[ot][s2] = frag_t(A2T, tile, OT, ot, s2);
                    o.tb[ot][s2] = frag_t(DOT, tile, OT, ot, s2);
                }
        }
    };
    Tile cur, nxt;
    const int n_tiles = slice_rows / 32;
    load_tile(0, cur, true, HALF == 1);
#pragma unroll 1
    for (int tl = 0; tl < n_tiles; ++tl) {
        if constexpr (HALF == 0) load_tile(tl, cur, false, true);
        if (tl + 1 < n_tiles) load_tile(tl + 1, nxt, true, HALF == 1);
        // register v of a "[row][hidden]" accumulator: row 8 (v / 4) + 4 h + v % 4 of the tile
        if constexpr (HALF == 0) {
            f32x16 a1, du2 = {0};
#pragma unroll
            for (int v = 0; v < 16; ++v) a1[v] = c1;
#pragma unroll
            for (int s = 0; s < KS; ++s) a1 = mfma32(cur.ra[s], wa[s], a1);
#pragma unroll
            for (int t = 0; t < RS; ++t) du2 = mfma32(cur.rb[t], wb[t], du2);
            f32x16 hh;
            // (one wave writes and reads its own part: the wave's LDS instructions complete in order)
            float *my = stl[wave];
            my[h * 32 + x] = cur.st[0];
            my[(2 + h) * 32 + x] = cur.st[1];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const f32x4 mu = *(const f32x4 *)&my[0 * 32 + 8 * g4 + 4 * h];
                const f32x4 iv = *(const f32x4 *)&my[1 * 32 + 8 * g4 + 4 * h];
                const f32x4 m1 = *(const f32x4 *)&my[2 * 32 + 8 * g4 + 4 * h];
                const f32x4 m2 = *(const f32x4 *)&my[3 * 32 + 8 * g4 + 4 * h];
#pragma unroll
                for (int j2 = 0; j2 < 4; ++j2) {
                    const int v = 4 * g4 + j2;
                    float y, dy;
                    gelu_and_slope(a1[v], y, dy);
                    const float hv = (y - mu[j2]) * iv[j2];
                    sg2 += du2[v] * hv;
                    sb2 += du2[v];
                    const float d = iv[j2] * (g2h * du2[v] - m1[j2] - hv * m2[j2]) * dy;
                    sda1 += d;
                    hh[v] = hv;
                    a1[v] = d;                              // da1
                }
            }
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const bf16x8 da1f = cvt8_from16(a1, 8 * s2), hhf = cvt8_from16(hh, 8 * s2);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) accA[dt] = mfma32(cur.ta[dt][s2], da1f, accA[dt]);
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) sda2[ot] += (float)cur.tb[ot][s2][e];
                    accB[ot] = mfma32(hhf, cur.tb[ot][s2], accB[ot]);
                }
            }
        } else {
            f32x16 a3 = {0}, dh3 = {0};
#pragma unroll
            for (int t = 0; t < RS; ++t) {
                a3 = mfma32(cur.ra[t], wa[t], a3);
                dh3 = mfma32(cur.rb[t], wb[t], dh3);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float y, dy;
                gelu_and_slope(a3[v], y, dy);
                a3[v] = y;                                  // h3
                dh3[v] *= dy;                               // da3
            }
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const bf16x8 h3f = cvt8_from16(a3, 8 * s2), da3f = cvt8_from16(dh3, 8 * s2);
#pragma unroll
                for (int ot = 0; ot < OT; ++ot) {
                    accA[ot] = mfma32(cur.ta[ot][s2], da3f, accA[ot]);
                    accB[ot] = mfma32(h3f, cur.tb[ot][s2], accB[ot]);
                }
            }
        }
        if constexpr (HALF == 0) {
#pragma unroll
            for (int s = 0; s < KS; ++s) cur.ra[s] = nxt.ra[s];
#pragma unroll
            for (int t = 0; t < RS; ++t) cur.rb[t] = nxt.rb[t];
            cur.st[0] = nxt.st[0];
            cur.st[1] = nxt.st[1];
        } else {
            cur = nxt;
        }
    }

    // ---- write this chunk's part of the slice's sums (blob layout, fp32) ----
    // register v of an accumulator: row i = 8 (v / 4) + 4 h + v % 4, lane x = column
    float *out = part + (size_t)slice * blob_len + Net::offset_of(net, 4);
    float *oW1 = out + 2 * D, *og2 = oW1 + (size_t)D * HID, *ob2 = og2 + HID, *oW2 = ob2 + HID;
    float *oW3 = oW2 + (size_t)HID * R, *oW4 = oW3 + (size_t)R * HID;
    if constexpr (HALF == 0) {
        sda1 += __shfl_xor(sda1, 32);
        sg2 += __shfl_xor(sg2, 32);
        sb2 += __shfl_xor(sb2, 32);
        if (h == 0) {
            og2[hid] = sg2;
            ob2[hid] = sb2;
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = 32 * dt + 8 * (v / 4) + 4 * h + v % 4;        // dW1[k][hid], u1 = g1 x^ + b1
                oW1[(size_t)k * HID + hid] = bf16_to_f32(nt.g1[k]) * accA[dt][v] + bf16_to_f32(nt.b1[k]) * sda1;
            }
#pragma unroll
        for (int ot = 0; ot < OT; ++ot) {
            const float s2all = sda2[ot] + __shfl_xor(sda2[ot], 32);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int hr = 32 * ch + 8 * (v / 4) + 4 * h + v % 4;       // dW2[hr][o], u2 = g2 h^ + b2
                oW2[(size_t)hr * R + 32 * ot + x] = bf16_to_f32(nt.g2[hr]) * accB[ot][v] + bf16_to_f32(nt.b2[hr]) * s2all;
            }
        }
        if (cg == 0 && wave == 0) {
            // dg1, db1: the row kernel's workgroup sums over this slice, in order
            const size_t wg0 = first / 256;
            for (int idx = lane; idx < 2 * D; idx += 64) {
                float sum = 0.f;
                for (int k = 0; k < slice_rows / 256; ++k) sum += GB1[((wg0 + k) * 2 + net) * 2 * D + idx];
                out[idx] = sum;
            }
        }
    } else {
#pragma unroll
        for (int ot = 0; ot < OT; ++ot)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 8 * (v / 4) + 4 * h + v % 4;
                oW4[(size_t)(32 * ch + i) * R + 32 * ot + x] = accB[ot][v];      // dW4[hidden][o]
                oW3[(size_t)(32 * ot + i) * HID + hid] = accA[ot][v];            // dW3[f][hid]
            }
    }
}

// Slices per unit for the parameter kernel: enough workgroups to fill the GPU several times over,
// slices of at least 512 rows that are multiples of 256.
int learned_bwd_slices(const Problem &pb)
{
    const int jobs = 2 * (pb.r / 4 / 4);
    int k = 1;
    while ((long long)pb.units * k * jobs < 2048 && pb.n / (2 * k) >= 512 && pb.n % (2 * k * 256) == 0) k *= 2;
    return k;
}

// dG[set][idx] = sum over the sides (query rows, key rows) and the slices of the units of the
// set, in order.  part: [side][unit][slice of the unit][blob].
__global__ __launch_bounds__(kWg) void k_learned_bwd_reduce(const float *__restrict__ part, float *__restrict__ dG,
                                                            size_t blob_len, int units, int per_unit, int heads,
                                                            int per_head)
{
    const size_t idx = (size_t)blockIdx.x * kWg + threadIdx.x;
    const int set = blockIdx.y;
    if (idx >= blob_len) return;
    const int step = per_head ? heads : 1;
    float sum = 0.f;
    // (the additions keep their order; the loads of up to eight slices are in flight together)
    for (int side = 0; side < 2; ++side)
        for (int u = per_head ? set : 0; u < units; u += step) {
            const float *src = part + (((size_t)side * units + u) * per_unit) * blob_len + idx;
            int k = 0;
            for (; k + 8 <= per_unit; k += 8) {
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = src[(size_t)(k + j) * blob_len];
#pragma unroll
                for (int j = 0; j < 8; ++j) sum += v[j];
            }
            for (; k < per_unit; ++k) sum += src[(size_t)k * blob_len];
        }
    dG[(size_t)set * blob_len + idx] = sum;
}

// m(K) as bf16 rows from the token octets [rows/8][2][R][4] fp32 the key-side sketch kernel writes.
template <int R>
__global__ __launch_bounds__(kWg) void k_octets_to_rows(const float *__restrict__ M8, bf16_t *__restrict__ M_rm,
                                                        size_t count4)
{
    const size_t idx = (size_t)blockIdx.x * kWg + threadIdx.x;  // ((oct * 2 + h) * R + col)
    if (idx >= count4) return;
    const f32x4 m4 = *(const f32x4 *)&M8[idx * 4];
    const size_t oh = idx / R;
    const int col = (int)(idx % R);
    const size_t tok = (oh / 2) * 8 + (oh % 2) * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) M_rm[(tok + j) * R + col] = f32_to_bf16(m4[j]);
}
